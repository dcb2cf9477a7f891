// C ABI of the AASD hot path: argument validation and kernel launches (see include/aasd.h).
// Validation touches no HIP API, so every error path can be exercised without a GPU.
#include "aasd.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "retrieve.hip.h"
#include "row_sweep.hip.h"
#include "verify_tail.hip.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

bool valid_dtype(int32_t dt) { return dt == AASD_F32 || dt == AASD_BF16; }
size_t elt_size(int32_t dt) { return dt == AASD_F32 ? 4 : 2; }

// Launch shape of the row sweep (threads per row, 16-byte loads in flight per lane and buffer).
// Measured on MI355X at V = 128256 bf16: without the LDS chunk-maximum array (verification) 1024
// threads x 2 loads is fastest at every row count; with it (alignment sampling) occupancy is
// LDS-bound and 256 x 4 wins.  The environment variable
// AASD_SWEEP_CONFIG="block,unroll" overrides the choice (developer knob for tuning and tests).
struct SweepConfig { int block, unroll; };

SweepConfig sweep_config(bool align, int64_t rows)
{
    SweepConfig cfg = align ? SweepConfig{256, 4} : SweepConfig{1024, 2};
    (void)rows;
    if (const char* e = getenv("AASD_SWEEP_CONFIG")) {
        int b = 0, u = 0;
        if (sscanf(e, "%d,%d", &b, &u) == 2) { cfg.block = b; cfg.unroll = u; }
    }
    return cfg;
}

constexpr size_t kMaxChunkMaxLds = 60 * 1024;      // dynamic LDS the sweep may use for chunk maxima
constexpr int64_t kMaxRowsPerLaunch = 1 << 22;     // keeps gridDim.x * blockDim.x below 2^32

template <int DT, bool ALIGN, bool COUNT, int BLOCK, int U>
hipError_t launch_sweep_one(const aasd::SweepParams& p, int64_t rows, size_t dyn_lds, hipStream_t stream)
{
    for (int64_t row0 = 0; row0 < rows; row0 += kMaxRowsPerLaunch) {
        const int64_t n = rows - row0 < kMaxRowsPerLaunch ? rows - row0 : kMaxRowsPerLaunch;
        hipLaunchKernelGGL((aasd::row_sweep_kernel<DT, ALIGN, COUNT, BLOCK, U>), dim3((unsigned)n), dim3(BLOCK),
                           dyn_lds, stream, p, row0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int DT, bool ALIGN, bool COUNT>
int launch_sweep(const aasd::SweepParams& p, int64_t rows, size_t dyn_lds, hipStream_t stream)
{
    const SweepConfig cfg = sweep_config(ALIGN, rows);
    hipError_t e;
    if (cfg.block == 256 && cfg.unroll == 4) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 4>(p, rows, dyn_lds, stream);
    else if (cfg.block == 256 && cfg.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 2>(p, rows, dyn_lds, stream);
    else if (cfg.block == 512 && cfg.unroll == 4) e = launch_sweep_one<DT, ALIGN, COUNT, 512, 4>(p, rows, dyn_lds, stream);
    else if (cfg.block == 512 && cfg.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 512, 2>(p, rows, dyn_lds, stream);
    else if (cfg.block == 256 && cfg.unroll == 8) e = launch_sweep_one<DT, ALIGN, COUNT, 256, 8>(p, rows, dyn_lds, stream);
    else if (cfg.block == 512 && cfg.unroll == 8) e = launch_sweep_one<DT, ALIGN, COUNT, 512, 8>(p, rows, dyn_lds, stream);
    else if (cfg.block == 1024 && cfg.unroll == 4) e = launch_sweep_one<DT, ALIGN, COUNT, 1024, 4>(p, rows, dyn_lds, stream);
    else if (cfg.block == 1024 && cfg.unroll == 2) e = launch_sweep_one<DT, ALIGN, COUNT, 1024, 2>(p, rows, dyn_lds, stream);
    else if (cfg.block == 1024 && cfg.unroll == 1) e = launch_sweep_one<DT, ALIGN, COUNT, 1024, 1>(p, rows, dyn_lds, stream);
    else return fail(AASD_ERR_UNSUPPORTED, "AASD_SWEEP_CONFIG=%d,%d is not a compiled launch shape", cfg.block, cfg.unroll);
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "row sweep launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

}  // namespace

extern "C" {

const char* aasd_version(void) { return "aasd-mi355x 0.1 (gfx950)"; }

const char* aasd_last_error(void) { return g_err; }

int aasd_align_sample(const void* logits, int32_t dt, int64_t rows, int32_t V, int64_t row_stride,
                      const int32_t* next_tok, int32_t m, int32_t c, int32_t mode, uint64_t seed,
                      uint64_t row_id_base, int32_t* argmax, uint8_t* misaligned, float* entropy,
                      float* p_next, float* p_max, int32_t* rank, int32_t* extras,
                      uint8_t* n_extras, uint32_t* near_count, void* stream)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "align_sample: unknown dtype %d", dt);
    if (rows < 0) return fail(AASD_ERR_INVALID_ARG, "align_sample: rows = %lld < 0", (long long)rows);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "align_sample: V = %d <= 0", V);
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "align_sample: row_stride %lld < V %d", (long long)row_stride, V);
    if (m < 0 || m > AASD_MAX_EXTRAS) return fail(AASD_ERR_INVALID_ARG, "align_sample: m = %d outside [0,%d]", m, AASD_MAX_EXTRAS);
    if (c < 1 || c < m || c > AASD_MAX_CANDSET)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: c = %d outside [max(m,1),%d]", c, AASD_MAX_CANDSET);
    if (mode != AASD_EXTRAS_TOP && mode != AASD_EXTRAS_SAMPLE)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: unknown mode %d", mode);
    if (rows == 0) return AASD_OK;
    if (!logits || !argmax || !misaligned || !entropy || !p_next || !p_max)
        return fail(AASD_ERR_INVALID_ARG, "align_sample: null required pointer");
    if (m > 0 && (!extras || !n_extras))
        return fail(AASD_ERR_INVALID_ARG, "align_sample: extras and n_extras are required when m > 0");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "align_sample: logits pointer is not aligned to its element size");

    aasd::SweepParams p{};
    p.logits = logits; p.V = V; p.row_stride = row_stride; p.seq_stride = row_stride; p.rows_per_seq = 1;
    p.next_tok = next_tok; p.m_x = m; p.c = c; p.mode = mode; p.seed = seed; p.row_id_base = row_id_base;
    p.argmax = argmax; p.misaligned = misaligned; p.entropy = entropy; p.p_next = p_next; p.p_max = p_max;
    p.rank = rank; p.extras = extras; p.n_extras = n_extras; p.near_count = near_count;

    // one chunk maximum per 16-byte vector of the row, kept in LDS when it fits
    size_t dyn = 0;
    if (m > 0 && next_tok) {
        const size_t per_vec = dt == AASD_BF16 ? 8 : 4;
        const size_t need = ((size_t)V / per_vec + 1) * elt_size(dt);
        if (need <= kMaxChunkMaxLds) { dyn = (need + 15) & ~(size_t)15; p.cm_enabled = 1; }
    }
    hipStream_t s = (hipStream_t)stream;
    if (dt == AASD_BF16) {
        return rank ? launch_sweep<AASD_BF16, true, true>(p, rows, dyn, s) : launch_sweep<AASD_BF16, true, false>(p, rows, dyn, s);
    }
    return rank ? launch_sweep<AASD_F32, true, true>(p, rows, dyn, s) : launch_sweep<AASD_F32, true, false>(p, rows, dyn, s);
}

int aasd_retrieve_drafts(const int32_t* tokens, int64_t tok_stride, const int32_t* len,
                         const int32_t* prompt_len, int32_t B, int32_t n_min, int32_t n_max,
                         int32_t k, int32_t C, const int32_t* extras, const uint8_t* n_extras,
                         int32_t m, int64_t extras_stride, int32_t* drafts, int32_t* draft_len,
                         int32_t* src_pos, int32_t* n_cand, int32_t* key_len,
                         int32_t* draft_extras, uint8_t* strict, void* stream)
{
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: B = %d < 0", B);
    if (tok_stride < 1) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: tok_stride = %lld < 1", (long long)tok_stride);
    if (tok_stride > 0x7fffffffLL) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: tok_stride exceeds int32");
    if (n_min < 1 || n_min > n_max || n_max > AASD_MAX_KEY)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: need 1 <= n_min <= n_max <= %d (got %d, %d)", AASD_MAX_KEY, n_min, n_max);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    const bool have_table = extras != nullptr || n_extras != nullptr;
    if (have_table && (!extras || !n_extras))
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: extras and n_extras must be given together");
    if (have_table && (m < 1 || m > AASD_MAX_EXTRAS))
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: m = %d outside [1,%d] with an alignment table", m, AASD_MAX_EXTRAS);
    if (have_table && extras_stride < 0) return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: extras_stride < 0");
    if (draft_extras && !have_table)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: draft_extras needs the alignment table");
    if (B == 0) return AASD_OK;
    if (!tokens || !len || !prompt_len || !drafts || !draft_len || !src_pos || !n_cand || !key_len || !strict)
        return fail(AASD_ERR_INVALID_ARG, "retrieve_drafts: null required pointer");

    aasd::RetrieveParams p{};
    p.tokens = tokens; p.tok_stride = tok_stride; p.len = len; p.prompt_len = prompt_len;
    p.B = B; p.n_min = n_min; p.n_max = n_max; p.k = k; p.C = C;
    p.extras = extras; p.n_extras = n_extras; p.m_x = have_table ? m : 0; p.extras_stride = extras_stride;
    p.drafts = drafts; p.draft_len = draft_len; p.src_pos = src_pos; p.n_cand = n_cand; p.key_len = key_len;
    p.draft_extras = draft_extras; p.strict = strict;
    // positions per lane per tile: enough for the whole buffer when it fits in 64 KB of LDS, odd
    constexpr int kMaxRun = 11;  // (8 + 1024*11) * 4 + 1024*11 = 56,352 bytes
    int run = (int)((tok_stride + aasd::kRetrieveBlock - 1) / aasd::kRetrieveBlock);
    if (run > kMaxRun) run = kMaxRun;
    run |= 1;
    p.run = run;
    p.tile = run * aasd::kRetrieveBlock;
    const size_t dyn = (size_t)(AASD_MAX_KEY + p.tile) * 4 + (size_t)p.tile;
    hipLaunchKernelGGL(aasd::retrieve_kernel, dim3((unsigned)B), dim3(aasd::kRetrieveBlock), dyn, (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "retrieve_drafts launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

size_t aasd_verify_workspace_bytes(int32_t B, int32_t C, int32_t k)
{
    if (B < 0 || C < 1 || C > AASD_MAX_CANDIDATES || k < 1 || k > AASD_MAX_DRAFT) return 0;
    return (size_t)B * (size_t)(1 + C * k) * sizeof(float4);
}

int aasd_verify(const void* logits, int32_t dt, int32_t B, int32_t C, int32_t k, int32_t V,
                int64_t row_stride, int64_t seq_stride, const int32_t* drafts,
                const int32_t* draft_len, const uint8_t* strict, float alpha, float beta,
                uint32_t flags, int32_t* accept_len, int32_t* best_cand, int32_t* next_token,
                float* row_entropy, float* row_pmax, int32_t* row_argmax, float* tok_p,
                float* tok_delta, uint32_t* near_count, void* workspace, size_t workspace_bytes,
                void* stream)
{
    if (!valid_dtype(dt)) return fail(AASD_ERR_INVALID_ARG, "verify: unknown dtype %d", dt);
    if (B < 0) return fail(AASD_ERR_INVALID_ARG, "verify: B = %d < 0", B);
    if (k < 1 || k > AASD_MAX_DRAFT) return fail(AASD_ERR_INVALID_ARG, "verify: k = %d outside [1,%d]", k, AASD_MAX_DRAFT);
    if (C < 1 || C > AASD_MAX_CANDIDATES) return fail(AASD_ERR_INVALID_ARG, "verify: C = %d outside [1,%d]", C, AASD_MAX_CANDIDATES);
    if (V <= 0) return fail(AASD_ERR_INVALID_ARG, "verify: V = %d <= 0", V);
    const int64_t R = 1 + (int64_t)C * k;
    if (row_stride < V) return fail(AASD_ERR_INVALID_ARG, "verify: row_stride %lld < V %d", (long long)row_stride, V);
    if (seq_stride < R * row_stride)
        return fail(AASD_ERR_INVALID_ARG, "verify: seq_stride %lld < R*row_stride %lld", (long long)seq_stride, (long long)(R * row_stride));
    if (flags & ~AASD_VERIFY_NO_CLAMP) return fail(AASD_ERR_INVALID_ARG, "verify: unknown flag bits 0x%x", flags);
    if (B == 0) return AASD_OK;
    if (!logits || !drafts || !draft_len || !accept_len || !best_cand || !next_token)
        return fail(AASD_ERR_INVALID_ARG, "verify: null required pointer");
    if (((uintptr_t)logits % elt_size(dt)) != 0)
        return fail(AASD_ERR_UNSUPPORTED, "verify: logits pointer is not aligned to its element size");
    const size_t need = aasd_verify_workspace_bytes(B, C, k);
    if (!workspace || workspace_bytes < need)
        return fail(AASD_ERR_WORKSPACE, "verify: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)workspace % 16) != 0) return fail(AASD_ERR_WORKSPACE, "verify: workspace is not 16-byte aligned");

    hipStream_t s = (hipStream_t)stream;
    aasd::SweepParams sp{};
    sp.logits = logits; sp.V = V; sp.row_stride = row_stride; sp.seq_stride = seq_stride; sp.rows_per_seq = (int32_t)R;
    sp.c = 1;
    sp.stats = (float4*)workspace; sp.row_entropy = row_entropy; sp.row_pmax = row_pmax; sp.row_argmax = row_argmax;
    const int64_t rows = (int64_t)B * R;
    int rc = dt == AASD_BF16 ? launch_sweep<AASD_BF16, false, false>(sp, rows, 0, s)
                             : launch_sweep<AASD_F32, false, false>(sp, rows, 0, s);
    if (rc != AASD_OK) return rc;

    aasd::VerifyTailParams tp{};
    tp.logits = logits; tp.B = B; tp.C = C; tp.k = k; tp.V = V; tp.row_stride = row_stride; tp.seq_stride = seq_stride;
    tp.drafts = drafts; tp.draft_len = draft_len; tp.strict = strict; tp.alpha = alpha; tp.beta = beta; tp.flags = flags;
    tp.accept_len = accept_len; tp.best_cand = best_cand; tp.next_token = next_token;
    tp.tok_p = tok_p; tp.tok_delta = tok_delta; tp.near_count = near_count; tp.stats = (const float4*)workspace;
    if (dt == AASD_BF16)
        hipLaunchKernelGGL(aasd::verify_tail_kernel<AASD_BF16>, dim3((unsigned)B), dim3(aasd::kTailBlock), 0, s, tp);
    else
        hipLaunchKernelGGL(aasd::verify_tail_kernel<AASD_F32>, dim3((unsigned)B), dim3(aasd::kTailBlock), 0, s, tp);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AASD_ERR_LAUNCH, "verify tail launch failed: %s", hipGetErrorString(e));
    return AASD_OK;
}

}  // extern "C"
