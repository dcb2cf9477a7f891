// Draft tree (Sec. 3.2, Eq. 2): merging the candidate n-grams and the alignment extras of their
// positions into one tree under the last committed token, the tree attention mask, and conditional
// verification (Sec. 3.3) over that tree.
#pragma once

#include "row_finish.hip.h"

namespace aasd {

constexpr int kTreeBlock = 256;
constexpr int kMaxLayerEvents = AASD_MAX_CANDIDATES * (1 + AASD_MAX_EXTRAS);  // 160 tokens can enter one layer

struct BuildTreeParams {
    const int32_t* drafts;        // [B, C, k]
    const int32_t* draft_len;     // [B, C]
    const uint8_t* strict;        // [B, C, k] or null
    const int32_t* draft_extras;  // [B, C, k, m] or null
    int32_t m_x;
    const int32_t* root_tok;      // [B] or null
    int32_t B, C, k, max_nodes;
    uint32_t w_magic;             // floor(2^32 / W) + 1 for W = ceil(max_nodes / 32) mask words per row (0 for W = 1)
    int32_t* node_token;
    int32_t* node_parent;
    int32_t* node_depth;
    uint8_t* node_strict;
    int32_t* n_nodes;
    uint32_t* mask;               // [B, max_nodes, W] or null
    int32_t* cand_node;           // [B, C, k] or null
};

// The layer loop of build_tree_kernel for a sequence whose events of one layer fit one wave (C * (1 + m) <= 64:
// the paper's 16 candidates with two extras each are 48).  One wave, a lane per event, no barrier and no LDS
// traffic between lanes except the nodes' own arrays.  The events of a layer are grouped by key, one group per
// trip of a loop: the lowest lane not yet grouped names a key (two lane reads), a ballot finds the lanes that
// share it, and since the trips go through the first events in ascending order the group's node is simply the
// next free one, which is the numbering of a serial insertion into a (parent, token) dictionary.  Every lane
// of a candidate keeps the node at the end of the candidate's path in a register.  The lane of a node's first
// event writes its mask row (the parent's row plus the node's own bit) with 16-byte LDS accesses.
// Same events, same order, same node numbers as the workgroup-wide loop of the kernel.  Returns the node count.
__device__ __forceinline__ int tree_layers_one_wave(int lane, int C, int k, int m, int N, int Wp,
                                                    const int* s_tok, const int* s_x, const unsigned char* s_strict,
                                                    const int* s_dl, int* s_cn, int* n_tok, int* n_par, int* n_dep,
                                                    unsigned char* n_str, uint32_t* n_mask)
{
    const int per = 1 + m, E = C * per;
    const int e = lane, c = e < E ? e / per : 0, slot = e - (e / per) * per;
    const int dl = e < E ? s_dl[c] : 0;
    const int own_lane = c * per;   // the lane of the candidate's own token (slot 0)
    // this lane's event of layer j: what it would add does not depend on where the candidate's path stands
    auto load_event = [&](int j, int& main_tok, int& x, int& st) {
        const bool have = e < E && j <= dl;
        const int at = c * k + (j - 1);
        main_tok = have ? s_tok[at] : -1;
        x = (have && slot > 0) ? s_x[at * m + (slot - 1)] : -1;
        st = (have && slot == 0) ? s_strict[at] : 0;   // extras are verified conditionally
    };
    int main_tok, x, st;
    load_event(1, main_tok, x, st);
    int cur = 0;                    // node at the end of the candidate's path; every path starts at the root
    int n = 1;
    for (int j = 1; j <= k; ++j) {
        const int par = cur;
        const int tok = slot == 0 ? main_tok : x;
        const int at = c * k + (j - 1);
        // a missing token ends the candidate's path, extras included
        const bool valid = e < E && j <= dl && par >= 0 && main_tok >= 0 && tok >= 0;
        const bool conditional_event = valid && st == 0;
        unsigned long long remaining = __ballot(valid);
        if (remaining == 0ull) break;   // no candidate reaches this layer
        const unsigned long long conditional = __ballot(conditional_event);
        if (j < k) load_event(j + 1, main_tok, x, st);   // the next layer's event, in flight behind this layer's work
        // Per trip the lanes do one select; everything else is kept in scalar masks and read out after the loop.
        int nid = -1, created = 0;
        unsigned long long firsts = 0ull, cond_groups = 0ull;
        while (remaining != 0ull) {   // one trip per distinct key of the layer
            const int L = __ffsll((long long)remaining) - 1;
            const int bpar = __builtin_amdgcn_readlane(par, L), btok = __builtin_amdgcn_readlane(tok, L);
            const bool in = valid && par == bpar && tok == btok;
            const unsigned long long grp = __ballot(in);
            if (in) nid = n + created < N ? n + created : -1;   // beyond the node budget: dropped
            firsts |= 1ull << L;
            if ((grp & conditional) != 0ull) cond_groups |= grp;   // one conditional source makes the node conditional
            remaining &= ~grp;
            ++created;
        }
        const bool first = ((firsts >> lane) & 1ull) != 0ull;
        const bool cond_node = ((cond_groups >> lane) & 1ull) != 0ull;
        const int cur_next = __shfl(nid, own_lane);   // the node of the candidate's own token; -1 if that is missing
        if (first && nid >= 0) {
            n_tok[nid] = tok; n_par[nid] = par; n_dep[nid] = j; n_str[nid] = cond_node ? 0 : 1;
            // the mask row: the parent's row (an earlier layer's) plus the node's own bit; rows are 16-byte aligned
            const u32x4* src = reinterpret_cast<const u32x4*>(n_mask + par * Wp);
            u32x4* dst = reinterpret_cast<u32x4*>(n_mask + nid * Wp);
            constexpr int kMaxQ = AASD_MAX_TREE_NODES / 128;
            u32x4 row[kMaxQ];
#pragma unroll
            for (int q = 0; q < kMaxQ; ++q)
                if (q * 4 < Wp) row[q] = src[q];
#pragma unroll
            for (int q = 0; q < kMaxQ; ++q)
                if (q * 4 < Wp) dst[q] = row[q];
            __hip_atomic_fetch_or(n_mask + nid * Wp + (nid >> 5), 1u << (nid & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
        cur = cur_next;   // -1 if the candidate's own token is missing: its path has ended
        if (valid && slot == 0) s_cn[at] = nid;
        n = n + created < N ? n + created : N;
        // One wave issues its LDS instructions in order, so the next layer's reads of these rows need no wait: the
        // fence only keeps the compiler from moving them.
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    }
    return n;
}

// One workgroup per sequence.  The candidates, their flags and their extras are first staged in LDS in one
// coalesced pass, so that the layer loop touches no global memory.  The tree grows layer by layer.  In layer j
// every (candidate, slot) pair is an event (slot 0 = the candidate's j-th token, slots 1..m = its extras) with
// the key (node at the end of the candidate's path, token).  An event whose key no earlier event of the
// layer has opens a node; nodes are numbered in event order, which is exactly the order a serial insertion
// into a (parent, token) dictionary would give.  The mask row of a new node is its parent's row plus its own
// bit.  A layer of at most 64 events is built by one wave (tree_layers_one_wave above); a larger one by a
// thread per event: the earliest event with the same key by an all-pairs compare over LDS, the numbers by a
// ballot/popcount prefix over the waves, with barriers between the phases.
__global__ __launch_bounds__(kTreeBlock) void build_tree_kernel(BuildTreeParams p)
{
    constexpr int kMaxW = AASD_MAX_TREE_NODES / 32;
    constexpr int kMaxCK = AASD_MAX_CANDIDATES * AASD_MAX_DRAFT;
    __shared__ int s_tok[kMaxCK];                       // drafts of this sequence
    __shared__ int s_x[kMaxCK * AASD_MAX_EXTRAS];       // their extras
    __shared__ unsigned char s_strict[kMaxCK];
    __shared__ int s_cn[kMaxCK];                        // node of every candidate token
    __shared__ int s_dl[AASD_MAX_CANDIDATES];
    __shared__ unsigned long long ev_key[kMaxLayerEvents];   // (parent + 1, token); events without a token get a key of their own
    __shared__ int ev_node[kMaxLayerEvents];
    __shared__ unsigned char ev_flag[kMaxLayerEvents];
    __shared__ int cur[AASD_MAX_CANDIDATES];
    __shared__ int n_tok[AASD_MAX_TREE_NODES], n_par[AASD_MAX_TREE_NODES], n_dep[AASD_MAX_TREE_NODES];
    __shared__ unsigned char n_str[AASD_MAX_TREE_NODES];
    __shared__ __align__(16) uint32_t n_mask[AASD_MAX_TREE_NODES * kMaxW];   // rows of Wp words (W rounded up to 4)
    __shared__ int wave_cnt[kTreeBlock / kWave];
    __shared__ int s_n;

    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int C = p.C, k = p.k, m = p.draft_extras ? p.m_x : 0, N = p.max_nodes;
    const int W = (N + 31) / 32, Wp = (W + 3) & ~3;
    const int per = 1 + m, E = C * per, CK = C * k;
    const int e = tid, c = e < E ? e / per : 0, slot = e - (e / per) * per;
    const size_t bck = (size_t)b * CK;

    for (int i = tid; i < CK; i += kTreeBlock) {
        s_tok[i] = p.drafts[bck + i];
        s_strict[i] = p.strict ? (p.strict[bck + i] != 0) : 0;
        s_cn[i] = -1;
    }
    for (int i = tid; i < CK * m; i += kTreeBlock) s_x[i] = p.draft_extras[bck * m + i];
    if (tid < C) {
        int dl = p.draft_len[(size_t)b * C + tid];
        s_dl[tid] = dl < 0 ? 0 : (dl > k ? k : dl);
        cur[tid] = 0;
    }
    if (tid == 0) {
        n_tok[0] = p.root_tok ? p.root_tok[b] : -1;
        n_par[0] = -1; n_dep[0] = 0; n_str[0] = 0;
    }
    if (tid < Wp) n_mask[tid] = tid == 0 ? 1u : 0u;   // the root sees itself
    __syncthreads();
    const int dl = e < E ? s_dl[c] : 0;

    int n = 1;  // nodes so far: the same value in every thread
    const bool one_wave = E <= kWave;
    if (one_wave) {   // the usual case: one wave builds the layers without a barrier
        if (wid == 0) {
            const int nn = tree_layers_one_wave(lane, C, k, m, N, Wp, s_tok, s_x, s_strict, s_dl, s_cn, n_tok, n_par, n_dep, n_str, n_mask);
            if (lane == 0) s_n = nn;
        }
        __syncthreads();
        n = s_n;
    }
    for (int j = 1; !one_wave && j <= k; ++j) {   // more events per layer than a wave has lanes: a thread per event, barriers between the phases
        bool valid = false;
        int tok = -1, par = -1, st = 0;
        if (e < E) {
            par = cur[c];
            if (par >= 0 && j <= dl) {
                const int at = c * k + (j - 1);
                const int main_tok = s_tok[at];
                if (main_tok >= 0) {  // a missing token ends the candidate's path, extras included
                    if (slot == 0) {
                        tok = main_tok; valid = true;
                        st = s_strict[at];
                    } else {
                        const int x = s_x[at * m + (slot - 1)];
                        if (x >= 0) { tok = x; valid = true; }  // extras are verified conditionally
                    }
                }
            }
            ev_key[e] = valid ? ((unsigned long long)(unsigned)(par + 1) << 32) | (unsigned)tok
                              : ((unsigned long long)(0x10000u + (unsigned)e) << 32);
            ev_flag[e] = (unsigned char)st;
        }
        if (__syncthreads_or(valid) == 0) break;   // no candidate reaches this layer: the tree is complete (same in every thread)
        int rep = e;  // earliest event of the layer with the same key (the loads do not depend on one another)
        if (valid) {
            const unsigned long long key = ev_key[e];
            for (int e2 = 0; e2 < E; ++e2)
                if (ev_key[e2] == key && e2 < rep) rep = e2;
        }
        const bool first = valid && rep == e;
        const unsigned long long bal = __ballot(first);
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wid] = __popcll(bal);
        __syncthreads();
        int offset = n, total = 0;
#pragma unroll
        for (int w = 0; w < kTreeBlock / kWave; ++w) {
            if (w < wid) offset += wave_cnt[w];
            total += wave_cnt[w];
        }
        int id = -1;
        if (first) {
            id = offset + before < N ? offset + before : -1;  // beyond the node budget: dropped
            ev_node[e] = id;
            if (id >= 0) {
                n_tok[id] = tok; n_par[id] = par; n_dep[id] = j;
                for (int wi = 0; wi < Wp; ++wi)   // the parent's row (an earlier layer) plus the node's own bit
                    n_mask[id * Wp + wi] = n_mask[par * Wp + wi] | ((id >> 5) == wi ? 1u << (id & 31) : 0u);
            }
        }
        __syncthreads();
        if (valid && !first && st == 0) ev_flag[rep] = 0;  // one conditional source makes the node conditional
        __syncthreads();
        if (first && id >= 0) n_str[id] = ev_flag[e];
        if (e < E && slot == 0) {
            const int nid = valid ? ev_node[rep] : -1;
            cur[c] = nid;
            if (valid) s_cn[c * k + (j - 1)] = nid;
        }
        n = n + total < N ? n + total : N;
        __syncthreads();
    }

    if (tid == 0) p.n_nodes[b] = n;
    for (int i = tid; i < N; i += kTreeBlock) {
        const size_t bi = (size_t)b * N + i;
        const bool used = i < n;
        p.node_token[bi] = used ? n_tok[i] : -1;
        p.node_parent[bi] = used ? n_par[i] : -1;
        p.node_depth[bi] = used ? n_dep[i] : 0;
        p.node_strict[bi] = used ? n_str[i] : 0;
    }
    if (p.mask)
        for (int i = tid; i < N * W; i += kTreeBlock) {
            const int q = (int)div_small((uint32_t)i, W, p.w_magic);   // node q, word i - q * W
            p.mask[(size_t)b * N * W + i] = q < n ? n_mask[q * Wp + (i - q * W)] : 0u;
        }
    if (p.cand_node)
        for (int i = tid; i < CK; i += kTreeBlock) p.cand_node[bck + i] = s_cn[i];
}

struct VerifyTreeParams {
    const void* logits;
    int32_t B, N, V;
    int64_t row_stride, seq_stride;
    const int32_t* node_token;
    const int32_t* node_parent;
    const uint8_t* node_strict;
    const int32_t* n_nodes;
    float alpha, beta;
    uint32_t flags;
    int32_t* accept_len;
    int32_t* best_node;
    int32_t* accept_path;  // [B, AASD_MAX_DRAFT]
    int32_t* next_token;
    float* node_p;
    float* node_delta;
    uint32_t* near_count;
    float* row_entropy;
    float* row_pmax;
    int32_t* row_argmax;
    const WavePartial* partials;  // [B * N][npart]
    int32_t npart;
};

// The decisions of one tree by one workgroup of NT threads.  Node i is decided against the row of its parent
// (Eq. 4-6); it is accepted iff it and all its ancestors pass; the deepest accepted node wins.
// (A one-launch form of sweep and decisions, as aasd_verify has, was built for trees too and measured no faster
// than the two kernels - here the arrival protocol costs what the second launch costs - so there is none.)
struct VerifyTreeShared {
    float4 stats[AASD_MAX_TREE_NODES];   // per row {max logit, S, H, bits of argmax}
    int par[AASD_MAX_TREE_NODES];
    unsigned char pass[AASD_MAX_TREE_NODES];
    unsigned char near[AASD_MAX_TREE_NODES];
    unsigned red_key[16], red_near[16];
};

template <int DT, int NT>
__device__ __forceinline__ void verify_tree_block(const VerifyTreeParams& p, int b, VerifyTreeShared& sh)
{
    static_assert(NT / kWave <= 16, "one reduction slot per wave");
    constexpr int kPer = (AASD_MAX_TREE_NODES + NT - 1) / NT;   // nodes per thread
    const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
    const int N = p.N;

    // Everything that does not depend on another load is asked for at once: the node count, and every node's
    // parent, token and flag (slots at or beyond the count are read and ignored).
    int par_r[kPer], tok_r[kPer];
    unsigned char st_r[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * NT;
        par_r[j] = -1; tok_r[j] = -1; st_r[j] = 0;
        if (i >= 1 && i < N) {
            const size_t bi = (size_t)b * N + i;
            par_r[j] = p.node_parent[bi];
            tok_r[j] = p.node_token[bi];
            if (p.node_strict) st_r[j] = p.node_strict[bi];
        }
    }
    int n = p.n_nodes[b];
    n = n < 1 ? 1 : (n > N ? N : n);

    // the logit of every node's token in its parent's row: in flight while the row statistics are put together
    float zt_r[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * NT;
        if (i >= n || par_r[j] < 0 || par_r[j] >= i) par_r[j] = -1;   // parents precede their children
        zt_r[j] = 0.f;
        if (par_r[j] >= 0 && tok_r[j] >= 0 && tok_r[j] < p.V)
            zt_r[j] = load_elt<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)par_r[j] * p.row_stride + tok_r[j]);
        if (i < N) sh.par[i] = par_r[j];
    }

    for (int r = n + tid; r < N; r += NT) {   // rows that are not in use
        const int64_t row = (int64_t)b * N + r;
        if (p.row_entropy) p.row_entropy[row] = 0.f;
        if (p.row_pmax) p.row_pmax[row] = 0.f;
        if (p.row_argmax) p.row_argmax[row] = -1;
    }

    // ---- statistics of the used rows from the sweep's partials: G lanes per row ----
    {
        int G = 1;
        while (G < p.npart) G <<= 1;
        const int rows_per_pass = NT / G;
        const int sub = tid / G, s = tid - sub * G;
        for (int r0 = 0; r0 < n; r0 += rows_per_pass) {
            const int r = r0 + sub;
            const bool have_row = r < n;
            const int64_t row = (int64_t)b * N + (have_row ? r : 0);
            WavePartial wp;
            wp.m = -INFINITY; wp.S = 0.f; wp.T = 0.f; wp.code = 0x7fffffff;
            if (have_row && s < p.npart) wp = p.partials[row * p.npart + s];
            const float m = group_reduce(wp.m, G, [](float x, float y) { return fmaxf(x, y); });
            const bool live = wp.S > 0.f;
            float dl2 = 0.f, f = 0.f;
            if (live) partial_scale(wp.m, m, dl2, f);
            const float S = group_reduce(live ? wp.S * f : 0.f, G, [](float x, float y) { return x + y; });
            const float T2 = group_reduce(live ? (wp.T + dl2 * wp.S) * f : 0.f, G, [](float x, float y) { return x + y; });
            const int code = group_reduce(live && wp.m == m ? wp.code : 0x7fffffff, G, [](int x, int y) { return min(x, y); });
            if (have_row && s == 0) {
                // the code names the chunk that holds the row's maximum; the greedy pick is found below, by a load that
                // is in flight while the nodes are decided (they do not need it)
                const float H = entropy_from_sums(S, T2);
                const float pmax = 1.0f / S;
                sh.stats[r] = make_float4(m, S, H, __int_as_float((unsigned)code < (unsigned)p.V ? code : -1));
                if (p.row_entropy) p.row_entropy[row] = H;
                if (p.row_pmax) p.row_pmax[row] = pmax;
            }
        }
    }
    __syncthreads();

    static_assert(kPer * NT >= AASD_MAX_TREE_NODES, "a thread per row as well");
    u32x4 am_chunk[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int r = tid + j * NT;
        am_chunk[j] = u32x4{0u, 0u, 0u, 0u};
        if (r < n) {
            const int code = __float_as_int(sh.stats[r].w);
            const RowShape rs = row_shape<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)r * p.row_stride, p.V);
            if (code >= rs.head && code < rs.tail0) am_chunk[j] = rs.vbase[(code - rs.head) / Elt<DT>::kPerVec];
        }
    }

    // ---- per-node decision against the parent's row ----
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * NT;
        if (i >= N) continue;
        const size_t bi = (size_t)b * N + i;
        const int par = par_r[j];
        bool pass = false, near = false;
        float pf = 0.f, df = 0.f;
        if (par >= 0) {
            const int t = tok_r[j];
            const float4 st = sh.stats[par];
            const double m = (double)st.x, S = (double)st.y, H = (double)st.z;
            const bool valid = t >= 0 && t < p.V;
            const float zt = zt_r[j];
            const double pr = valid ? exp((double)zt - m) / S : 0.0;
            const double Delta = 1.0 / S;                              // Eq. 6
            const double thr = (double)p.alpha * H + (double)p.beta;   // Eq. 5
            double delta;
            if (p.flags & AASD_VERIFY_NO_CLAMP) {
                delta = thr;
                pass = valid && pr >= delta;
            } else {
                delta = st_r[j] ? Delta : fmin(thr, Delta);
                pass = valid && (pr >= delta || zt == st.x);           // Eq. 4; ties with the maximum pass
            }
            near = fabs(pr - delta) < 1e-6;
            pf = (float)pr;
            df = (float)delta;
        }
        sh.pass[i] = pass;
        sh.near[i] = near;
        if (p.node_p) p.node_p[bi] = pf;
        if (p.node_delta) p.node_delta[bi] = df;
    }
    // the rows' greedy picks: the first element of the chunk that equals the maximum
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int r = tid + j * NT;
        if (r < n) {
            const int code = __float_as_int(sh.stats[r].w);
            int am = code < 0 ? 0 : code;
            const RowShape rs = row_shape<DT>(p.logits, (int64_t)b * p.seq_stride + (int64_t)r * p.row_stride, p.V);
            if (code >= rs.head && code < rs.tail0) {
                float z[Elt<DT>::kPerVec];
                unpack<DT>(am_chunk[j], z);
                const float m = sh.stats[r].x;
#pragma unroll
                for (int e = Elt<DT>::kPerVec - 1; e >= 0; --e)
                    if (z[e] == m) am = code + e;
            }
            sh.stats[r].w = __int_as_float(am);
            if (p.row_argmax) p.row_argmax[(int64_t)b * N + r] = am;
        }
    }
    __syncthreads();

    // ---- accepted iff the node and all its ancestors pass; depth by walking up (parents have smaller indices) ----
    int key = 0;
    unsigned nr = 0u;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = tid + j * NT;
        const int par = par_r[j];
        if (i >= N || par < 0) continue;
        bool reached = true;  // all ancestors pass: the node is evaluated
        int depth = 1;
        for (int a = par; a > 0; a = sh.par[a]) {
            reached = reached && sh.pass[a];
            ++depth;
        }
        if (reached && sh.pass[i]) key = max(key, (depth << 16) | (0xffff - i));  // deepest, then lowest index
        if (reached && sh.near[i]) ++nr;
    }
    key = wave_max(key);
    nr = wave_sum(nr);
    if (lane == 0) { sh.red_key[wid] = (unsigned)key; sh.red_near[wid] = nr; }
    __syncthreads();
    if (tid == 0) {
        unsigned best_key = 0, near_total = 0;
        for (int w = 0; w < NT / kWave; ++w) { best_key = max(best_key, sh.red_key[w]); near_total += sh.red_near[w]; }
        const int best = best_key ? (int)(0xffff - (best_key & 0xffff)) : 0;
        const int best_depth = (int)(best_key >> 16);
        p.accept_len[b] = best_depth;
        p.best_node[b] = best;
        p.next_token[b] = __float_as_int(sh.stats[best].w);
        if (p.near_count) p.near_count[b] = near_total;
        if (p.accept_path) {
            for (int d = 0; d < AASD_MAX_DRAFT; ++d) p.accept_path[(size_t)b * AASD_MAX_DRAFT + d] = -1;
            int d = best_depth;
            for (int a = best; a > 0; a = sh.par[a], --d)
                if (d >= 1 && d <= AASD_MAX_DRAFT) p.accept_path[(size_t)b * AASD_MAX_DRAFT + d - 1] = a;
        }
    }
}

// One workgroup per sequence; many lanes so that the partials of a large tree arrive in few rounds of loads.
constexpr int kVerifyTreeBlock = 1024;

template <int DT>
__global__ __launch_bounds__(kVerifyTreeBlock) void verify_tree_kernel(VerifyTreeParams p)
{
    __shared__ VerifyTreeShared sh;
    verify_tree_block<DT, kVerifyTreeBlock>(p, blockIdx.x, sh);
}

}  // namespace aasd
