// The denoiser handle, the batched DiT forward and the draft-and-refine loop.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "common.h"
#include "../../include/drf_measure.h"

using namespace drf;

namespace {

constexpr int kTFreq = 256;
constexpr int kMaxSlots = 65535;        // slots of one pass (some launches index slots by a grid dimension)
constexpr int kCondChunkRows = 1024;    // modulation-table rows kept at a time when a call has more
constexpr size_t kMaxGraphs = 8;        // captured drf_sample launch sequences kept per handle

struct LinearW {
    const float* w32 = nullptr;     // fp32 path weights [N][K]
    const bf16_t* w16 = nullptr;    // bf16 path weights [N][K]
    const float* b = nullptr;       // bias [N] fp32
    int N = 0, K = 0;
};

struct BlockW { LinearW qkv, proj, xq, xkv, xo, fc1, fc2; };

// Device buffers of one batched pass beyond the caller's inputs and outputs: activations, the
// conditioning front-end's rows and the modulation table, the K/V of a text context.  Either owned by
// the handle (grown on demand) or carved out of the library's static scratch array.
struct Workspace {
    float *resid = nullptr, *mod = nullptr, *cact32 = nullptr, *cscratch = nullptr;
    void *hbuf = nullptr, *qkv = nullptr, *mid = nullptr, *ybuf = nullptr, *ybuf2 = nullptr, *cact = nullptr;
    void *xkv = nullptr, *ctx_act = nullptr;    // cross-attention K/V cache [L][rows][ctx_len][2D] and its staging
    float* skpart = nullptr;                    // partial tiles of the split-K GEMM (bf16 path), or NULL: no split
};

// Arguments that fix the launch sequence of a drf_sample call, and the graph captured for them.
struct SampleKey {
    drf_sched_config sched; int mode, n, batch; const void *x_T, *cond, *null_cond, *x_0, *z; float cfg_scale;
    int has_noise; uint64_t seed; uint32_t field0; unsigned ws_gen;
};
struct GraphEntry {
    SampleKey key; hipGraphExec_t exec = nullptr; bool failed = false; unsigned long long last_use = 0;
};

struct Prof {
    int on = 0;                     // 0 off | 1 per launch | 2 per predictor pass of drf_sample
    std::vector<hipEvent_t> pool;
    struct Rec { int fam; size_t e0, e1; double work; };
    std::vector<Rec> recs;
    size_t used = 0;
};

}  // namespace

struct drf_denoiser {
    drf_dit_config cfg{};
    DitDims dm{};
    bool bf16 = false;
    int n_mod = 0;                  // 6 L D + 2 D modulation columns per slot
    std::vector<void*> allocs;      // everything freed at destroy
    // parameters on the device
    float* params32 = nullptr;      // the whole flat array (rounded to bf16 values in bf16 mode)
    const float *patch_w = nullptr, *patch_b = nullptr, *t_w1 = nullptr, *t_b1 = nullptr, *t_w2 = nullptr,
                *t_b2 = nullptr, *c_w = nullptr, *c_b = nullptr, *table = nullptr, *fin_w = nullptr, *fin_b = nullptr;
    LinearW ada;                    // all blocks' adaLN projections and the final one, stacked [n_mod][D]
    std::vector<BlockW> blk;
    float* pos = nullptr;           // [T][D]
    // workspace (owned)
    Workspace ws;
    int cap_slots = 0, cap_cond_rows = 0, cap_ctx_rows = 0;
    // sampler buffers
    int cap_sample_n = 0, cap_sample_g = 0;
    size_t cap_sample_field = 0;
    float *drafts = nullptr, *epsbuf = nullptr, *anchor = nullptr;
    void* cond_cat = nullptr; size_t cond_cat_bytes = 0;
    Prof prof;
    // the stream of this handle's last call and an event recorded behind that call's work
    hipStream_t last_stream = nullptr;
    hipEvent_t done = nullptr;
    // captured launch sequences of drf_sample calls (see graph_for_call)
    int graph_mode = 1;             // 0 never | 1 capture at the second call with the same arguments | 2 at the first
    unsigned ws_gen = 0;            // bumped whenever a buffer that launches point into is re-allocated
    hipStream_t cap_stream = nullptr;
    std::vector<GraphEntry> graphs;
    unsigned long long graph_clock = 0;
    long long graph_replays = 0;
};

namespace {

drf_status dev_alloc(drf_denoiser* d, void** p, size_t bytes)
{
    *p = nullptr;
    if (bytes == 0) bytes = 16;
    if (hipMalloc(p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        DRF_FAIL(DRF_ENOMEM, "device allocation of %zu bytes failed", bytes);
    }
    d->allocs.push_back(*p);
    return DRF_OK;
}

// Frees *pp and clears it, so that a later failure never leaves a freed address behind.
template <typename T> void dev_free(drf_denoiser* d, T** pp)
{
    void* p = (void*)*pp;
    *pp = nullptr;
    if (!p) return;
    for (size_t i = 0; i < d->allocs.size(); ++i)
        if (d->allocs[i] == p) { d->allocs.erase(d->allocs.begin() + (long)i); break; }
    (void)hipFree(p);
}

drf_status check_config(const drf_dit_config* c)
{
    if (!c) DRF_FAIL(DRF_EINVAL, "config is NULL");
    if (c->depth < 0 || c->hidden < 4 || c->heads < 1 || c->mlp_ratio < 1 || c->patch < 1 || c->in_ch < 1 ||
        c->lat_h < 1 || c->lat_w < 1)
        DRF_FAIL(DRF_EINVAL, "non-positive DiT dimension");
    if (c->dtype != DRF_F32 && c->dtype != DRF_BF16) DRF_FAIL(DRF_EINVAL, "unknown dtype");
    if (c->cond != DRF_COND_VECTOR && c->cond != DRF_COND_CLASS && c->cond != DRF_COND_TEXT) DRF_FAIL(DRF_EINVAL, "unknown cond kind");
    if (c->cond_dim < 1) DRF_FAIL(DRF_EINVAL, "cond_dim must be >= 1");
    if (c->cond == DRF_COND_TEXT ? c->ctx_len < 1 : c->ctx_len != 0) DRF_FAIL(DRF_EINVAL, "ctx_len must be >= 1 for text and 0 otherwise");
    if (c->hidden % c->heads || c->hidden % 4 || c->lat_h % c->patch || c->lat_w % c->patch)
        DRF_FAIL(DRF_ESHAPE, "need hidden %% heads == 0, hidden %% 4 == 0 and latent divisible by patch");
    const int d = c->hidden / c->heads;
    if (c->dtype == DRF_BF16) {
        if (c->hidden % 64 || d % 8 || d > 96) DRF_FAIL(DRF_ESHAPE, "bf16 needs hidden %% 64 == 0, head dim %% 8 == 0 and <= 96");
        if (c->cond == DRF_COND_TEXT && c->cond_dim % 64) DRF_FAIL(DRF_ESHAPE, "bf16 text conditioning needs cond_dim %% 64 == 0");
    } else if (d > 128) {
        DRF_FAIL(DRF_ESHAPE, "fp32 needs head dim <= 128");
    }
    if (c->hidden > 2048) DRF_FAIL(DRF_ESHAPE, "hidden must be <= 2048");
    return DRF_OK;
}

size_t weight_count(const drf_dit_config* c)
{
    const size_t D = (size_t)c->hidden, P = (size_t)c->in_ch * c->patch * c->patch, R = (size_t)c->mlp_ratio;
    size_t n = D * P + D + D * kTFreq + D + D * D + D;
    if (c->cond == DRF_COND_VECTOR) n += D * (size_t)c->cond_dim + D;
    else if (c->cond == DRF_COND_CLASS) n += ((size_t)c->cond_dim + 1) * D;
    size_t per = 6 * D * D + 6 * D + 3 * D * D + 3 * D + D * D + D + R * D * D + R * D + D * R * D + D;
    if (c->cond == DRF_COND_TEXT) per += D * D + D + 2 * D * (size_t)c->cond_dim + 2 * D + D * D + D;
    n += per * (size_t)c->depth;
    n += 2 * D * D + 2 * D + P * D + P;
    return n;
}

// round-to-nearest-even to bf16, kept in fp32
inline float rne_bf16(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    std::memcpy(&f, &u, 4);
    return f;
}

struct ProfScope {
    drf_denoiser* d; hipStream_t st; bool live = false; size_t rec = 0;
    ProfScope(drf_denoiser* d_, hipStream_t st_, int fam, double work) : d(d_), st(st_)
    {
        Prof& p = d->prof;
        const bool pass_family = fam == DRF_PROF_PASS_FULL || fam == DRF_PROF_PASS_OTHER;
        if (p.on == 0 || (p.on == 2) != pass_family) return;
        while (p.pool.size() < p.used + 2) {
            hipEvent_t ev;
            if (hipEventCreate(&ev) != hipSuccess) return;
            p.pool.push_back(ev);
        }
        live = true;
        p.recs.push_back({ fam, p.used, p.used + 1, work });
        rec = p.recs.size() - 1;
        (void)hipEventRecord(p.pool[p.used], st);
        p.used += 2;
    }
    ~ProfScope() { if (live) (void)hipEventRecord(d->prof.pool[d->prof.recs[rec].e1], st); }
};

// Sizes (bytes) of the Workspace members for a pass of `slots` slots, `cond_rows` conditioning rows and
// `ctx_rows` distinct text contexts: one table both the owned and the static workspace are built from.
struct WorkspaceBytes { size_t resid, hbuf, qkv, mid, ybuf, ybuf2, mod, cact32, cscratch, cact, xkv, ctx_act; };
WorkspaceBytes workspace_bytes(const drf_denoiser* d, size_t slots, size_t cond_rows, size_t ctx_rows)
{
    const size_t M = slots * d->dm.T, D = (size_t)d->dm.D, act = d->bf16 ? 2 : 4;
    WorkspaceBytes b{};
    b.resid = M * D * 4; b.hbuf = M * D * act; b.qkv = M * 3 * D * act; b.mid = M * (size_t)d->dm.R * D * act;
    b.ybuf = M * D * act; b.ybuf2 = d->bf16 ? M * D * act : 0;
    b.mod = cond_rows * d->n_mod * 4; b.cact32 = cond_rows * D * 4; b.cscratch = cond_rows * (kTFreq + 3 * D) * 4;
    b.cact = cond_rows * D * act;
    if (d->cfg.cond == DRF_COND_TEXT) {
        const size_t rl = ctx_rows * d->cfg.ctx_len;
        b.xkv = (size_t)d->dm.L * rl * 2 * D * act; b.ctx_act = rl * d->cfg.cond_dim * act;
    }
    return b;
}

// Activation buffers for `slots` samples per pass.  On a failed allocation every member is either a
// live buffer or NULL and the capacity is 0, so the handle stays usable.
drf_status ensure_workspace(drf_denoiser* d, int slots, hipStream_t st)
{
    if (slots <= d->cap_slots) return DRF_OK;
    DRF_HIP(hipStreamSynchronize(st));
    Workspace& w = d->ws;
    d->cap_slots = 0;
    ++d->ws_gen;
    dev_free(d, &w.resid); dev_free(d, &w.hbuf); dev_free(d, &w.qkv); dev_free(d, &w.mid); dev_free(d, &w.ybuf); dev_free(d, &w.ybuf2);
    const WorkspaceBytes b = workspace_bytes(d, (size_t)slots, 0, 0);
    drf_status rc;
    if (d->bf16 && !w.skpart && (rc = dev_alloc(d, (void**)&w.skpart, gemm_splitk_scratch_bytes())) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, (void**)&w.resid, b.resid)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.hbuf, b.hbuf)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.qkv, b.qkv)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.mid, b.mid)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.ybuf, b.ybuf)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.ybuf2, b.ybuf2)) != DRF_OK) return rc;
    d->cap_slots = slots;
    return DRF_OK;
}

// Conditioning buffers for `rows` slot rows: front-end scratch, SiLU(c), and the modulation table.
drf_status ensure_cond(drf_denoiser* d, int rows, hipStream_t st)
{
    if (rows <= d->cap_cond_rows) return DRF_OK;
    DRF_HIP(hipStreamSynchronize(st));
    Workspace& w = d->ws;
    d->cap_cond_rows = 0;
    ++d->ws_gen;
    dev_free(d, &w.mod); dev_free(d, &w.cact32); dev_free(d, &w.cscratch); dev_free(d, &w.cact);
    const WorkspaceBytes b = workspace_bytes(d, 0, (size_t)rows, 0);
    drf_status rc;
    if ((rc = dev_alloc(d, (void**)&w.mod, b.mod)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, (void**)&w.cact32, b.cact32)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, (void**)&w.cscratch, b.cscratch)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.cact, b.cact)) != DRF_OK) return rc;
    d->cap_cond_rows = rows;
    return DRF_OK;
}

drf_status ensure_ctx(drf_denoiser* d, int rows, hipStream_t st)
{
    if (d->cfg.cond != DRF_COND_TEXT || rows <= d->cap_ctx_rows) return DRF_OK;
    DRF_HIP(hipStreamSynchronize(st));
    Workspace& w = d->ws;
    d->cap_ctx_rows = 0;
    ++d->ws_gen;
    dev_free(d, &w.xkv); dev_free(d, &w.ctx_act);
    const WorkspaceBytes b = workspace_bytes(d, 0, 0, (size_t)rows);
    drf_status rc;
    if ((rc = dev_alloc(d, &w.xkv, b.xkv)) != DRF_OK) return rc;
    if ((rc = dev_alloc(d, &w.ctx_act, b.ctx_act)) != DRF_OK) return rc;
    d->cap_ctx_rows = rows;
    return DRF_OK;
}

drf_status gemm(drf_denoiser* d, const void* A, const LinearW& w, int M, Epilogue e, hipStream_t st, float* splitk_scratch = nullptr)
{
    e.bias = w.b;
    ProfScope ps(d, st, DRF_PROF_GEMM, 2.0 * M * (double)w.N * w.K);
    if (d->bf16) return launch_gemm_bf16((const bf16_t*)A, w.w16, M, w.N, w.K, e, st, 0, splitk_scratch);
    return launch_gemm_f32((const float*)A, w.w32, M, w.N, w.K, e, st);
}

Epilogue epi_store(void* out, int ldo, bool f32, bool gelu = false)
{
    Epilogue e{};
    e.mode = gelu ? EPI_STORE_GELU : EPI_STORE; e.out = out; e.ldo = ldo; e.out_f32 = f32 ? 1 : 0;
    return e;
}

Epilogue epi_heads(void* out, int M, const DitDims& dm)
{
    Epilogue e{};
    e.mode = EPI_STORE_HEADS; e.out = out; e.ldo = 3 * dm.D; e.out_f32 = 0;
    set_rows_per_slot(&e, dm.T);
    e.hid = dm.D; e.hd = dm.d; e.heads = dm.heads; e.plane = (size_t)M * dm.D;
    make_fast_div(dm.D, &e.hid_magic, &e.hid_shift);
    make_fast_div(dm.d, &e.hd_magic, &e.hd_shift);
    return e;
}

// bf16 branch output gate * (acc + bias), to be added to the residual stream by the next LayerNorm launch
Epilogue epi_gated(void* out, int ldo, const float* gate, int gate_ld, int rows_per_slot)
{
    Epilogue e{};
    e.mode = EPI_STORE_GATED; e.out = out; e.ldo = ldo; e.out_f32 = 0; e.gate = gate; e.gate_ld = gate_ld;
    set_rows_per_slot(&e, rows_per_slot);
    return e;
}

Epilogue epi_resid(float* resid, int ldo, const float* gate, int gate_ld, int rows_per_slot)
{
    Epilogue e{};
    e.mode = EPI_RESID; e.out = resid; e.ldo = ldo; e.out_f32 = 1; e.gate = gate; e.gate_ld = gate_ld;
    set_rows_per_slot(&e, rows_per_slot);
    return e;
}

// Asks a bf16 GEMM launch to warm the caches with the weights of a later one (see Epilogue::warm).
Epilogue with_warm(Epilogue e, const LinearW* next)
{
    if (next && next->w16) { e.warm = next->w16; e.warm_lines = (uint32_t)(((size_t)next->N * next->K * 2) / 128); }
    return e;
}

// K/V of the text context for every block: xkv[l][row][ctx][2D] = Linear(ctx[row]).
drf_status compute_ctx_kv(drf_denoiser* d, const Workspace& ws, const float* ctx, int rows, hipStream_t st)
{
    drf_status rc;
    const size_t rl = (size_t)rows * d->cfg.ctx_len, act = d->bf16 ? 2 : 4;
    const void* A = ctx;
    if (d->bf16) {
        ProfScope ps(d, st, DRF_PROF_ELEMWISE, 6.0 * rl * d->cfg.cond_dim);
        if ((rc = launch_f32_to_bf16(ctx, (bf16_t*)ws.ctx_act, rl * d->cfg.cond_dim, st)) != DRF_OK) return rc;
        A = ws.ctx_act;
    }
    for (int l = 0; l < d->dm.L; ++l) {
        void* out = (char*)ws.xkv + (size_t)l * rl * 2 * d->dm.D * act;
        if ((rc = gemm(d, A, d->blk[l].xkv, (int)rl, epi_store(out, 2 * d->dm.D, !d->bf16), st)) != DRF_OK) return rc;
    }
    return DRF_OK;
}

// Conditioning of `rows` slot rows (they need not belong to one pass): c = MLP(femb(tau)) + cond
// embedding per row, then every block's shift / scale / gate and the final layer's in ONE GEMM
// against the stacked adaLN projections.  Row r of the result is mod_out[r][0 .. n_mod).
drf_status conditioning(drf_denoiser* d, const Workspace& ws, const SlotMap& map, const void* cond, int rows, int row0,
                        float* mod_out, hipStream_t st)
{
    const int D = d->dm.D;
    drf_status rc;
    CondArgs ca{};
    ca.t_w1 = d->t_w1; ca.t_b1 = d->t_b1; ca.t_w2 = d->t_w2; ca.t_b2 = d->t_b2; ca.c_w = d->c_w; ca.c_b = d->c_b;
    ca.table = d->table; ca.cond = cond; ca.cond_kind = d->cfg.cond; ca.cond_dim = d->cfg.cond_dim; ca.D = D;
    ca.slots = rows; ca.map = map;
    ca.act_f32 = ws.cact32 + (size_t)row0 * D;
    ca.act_bf16 = d->bf16 ? (bf16_t*)ws.cact + (size_t)row0 * D : nullptr;
    ca.scratch = ws.cscratch + (size_t)row0 * (kTFreq + 3 * D);
    {
        ProfScope ps(d, st, DRF_PROF_ELEMWISE, 4.0 * rows * ((double)kTFreq * D + (double)D * D));
        if ((rc = launch_cond_embed(ca, st)) != DRF_OK) return rc;
    }
    const void* A = d->bf16 ? (const void*)ca.act_bf16 : (const void*)ca.act_f32;
    return gemm(d, A, d->ada, rows, epi_store(mod_out, d->n_mod, true), st);
}

// The batched forward on the buffers of `ws` (sized for at least `slots` slots by the caller).
// mod: this pass's rows of the modulation table (see conditioning()).
drf_status forward(drf_denoiser* d, const Workspace& ws, const float* x, const SlotMap& map, const float* mod, int slots,
                   int n_blocks, float* eps_out, float* resid_out, hipStream_t st)
{
    const DitDims& dm = d->dm;
    const int D = dm.D, M = slots * dm.T, nm = d->n_mod;
    const bool f32 = !d->bf16;
    drf_status rc;
    {
        ProfScope ps(d, st, DRF_PROF_ELEMWISE, (double)M * D * 8.0 + (double)M * dm.P * 4.0);
        if ((rc = launch_patch_embed(x, map, d->patch_w, d->patch_b, d->pos, dm, slots, ws.resid, st)) != DRF_OK) return rc;
    }
    const double ln_bytes = (double)M * D * (4.0 + (f32 ? 4.0 : 2.0));
    const size_t act = f32 ? 4 : 2;
    // bf16 path: the gated branch outputs (attention projection, MLP) are written as bf16 and added to
    // the fp32 residual stream by a LayerNorm launch that reads the stream anyway, instead of a
    // read-modify-write of the stream in the GEMM epilogue (where it cannot overlap the MFMA loop).
    // The stream is stored once per block, not twice: the LayerNorm before the MLP normalises
    // resid + attention output without storing it, and the first LayerNorm of the next block adds both
    // outputs, (resid + attention) + MLP in that order, and stores.  pend1 / pend2 are the outputs not
    // yet in the stored stream.  The last block's MLP updates the stream directly, so the LayerNorm
    // before it stores; so does the one before text cross-attention, whose projection does the same.
    // Every pass streams all block weights from HBM (they do not fit the caches between passes), and a
    // GEMM whose k-loop waits on first-touch weight lines runs measurably slower than the same GEMM with
    // warm weights.  So each bf16 GEMM of the block chain (qkv -> proj -> fc1 -> fc2 -> next block's
    // qkv) touches the weights of its successor while its own last round of tiles starts.
    const bf16_t *pend1 = nullptr, *pend2 = nullptr;
    const bool text = d->cfg.cond == DRF_COND_TEXT;
    auto ln = [&](const float* shift, const float* scale, int mod_ld, bool store) -> drf_status {
        const int n_add = (pend1 ? 1 : 0) + (pend2 ? 1 : 0);
        ProfScope ps(d, st, DRF_PROF_ELEMWISE, ln_bytes + (double)M * D * (2.0 * n_add + (n_add && store ? 4.0 : 0.0)));
        const drf_status r = launch_ln_modulate(ws.resid, pend1, pend2, store, shift, scale, mod_ld, dm.T, M, D, ws.hbuf, f32, st);
        if (store) pend1 = pend2 = nullptr;
        return r;
    };
    for (int l = 0; l < n_blocks; ++l) {
        const BlockW& b = d->blk[l];
        const float* mrow = mod + (size_t)l * 6 * D;        // shift1 | scale1 | gate1 | shift2 | scale2 | gate2
        if ((rc = ln(mrow, mrow + D, nm, true)) != DRF_OK) return rc;
        // bf16: q | k | v are stored head-major ([slot][head][token][d] planes) so that attention reads
        // whole contiguous tiles; fp32: packed rows
        if ((rc = gemm(d, ws.hbuf, b.qkv, M, f32 ? epi_store(ws.qkv, 3 * D, true) : with_warm(epi_heads(ws.qkv, M, dm), &b.proj), st, ws.skpart)) != DRF_OK) return rc;
        {
            AttnArgs aa{};
            aa.q = ws.qkv; aa.out = ws.hbuf; aa.ldo = D; aa.Nq = dm.T; aa.Nk = dm.T; aa.heads = dm.heads; aa.d = dm.d;
            aa.slots = slots; aa.kv_mod = 0;
            if (f32) {
                aa.k = (char*)ws.qkv + (size_t)D * act; aa.v = (char*)ws.qkv + (size_t)2 * D * act;
                aa.ldq = aa.ldk = 3 * D;
                aa.q_slot_stride = aa.kv_batch_stride = (size_t)dm.T * 3 * D; aa.q_head_stride = aa.kv_head_stride = dm.d;
            } else {
                aa.k = (char*)ws.qkv + (size_t)M * D * act; aa.v = (char*)ws.qkv + (size_t)2 * M * D * act;
                aa.ldq = aa.ldk = dm.d;
                aa.q_slot_stride = aa.kv_batch_stride = (size_t)dm.T * D; aa.q_head_stride = aa.kv_head_stride = (size_t)dm.T * dm.d;
            }
            ProfScope ps(d, st, DRF_PROF_ATTN, 4.0 * slots * dm.heads * (double)dm.T * dm.T * dm.d);
            if ((rc = f32 ? launch_attn_f32(aa, st) : launch_attn_bf16(aa, st)) != DRF_OK) return rc;
        }
        if (f32) {
            if ((rc = gemm(d, ws.hbuf, b.proj, M, epi_resid(ws.resid, D, mrow + 2 * D, nm, dm.T), st)) != DRF_OK) return rc;
        } else {
            if ((rc = gemm(d, ws.hbuf, b.proj, M, with_warm(epi_gated(ws.ybuf, D, mrow + 2 * D, nm, dm.T), text ? nullptr : &b.fc1), st, ws.skpart)) != DRF_OK) return rc;
            pend1 = (const bf16_t*)ws.ybuf;
        }
        if (d->cfg.cond == DRF_COND_TEXT) {
            const int ctx_rows = map.cond_mod ? map.cond_mod : slots;
            if ((rc = ln(nullptr, nullptr, 0, true)) != DRF_OK) return rc;
            if ((rc = gemm(d, ws.hbuf, b.xq, M, epi_store(ws.qkv, D, f32), st)) != DRF_OK) return rc;
            const char* kv = (const char*)ws.xkv + (size_t)l * ctx_rows * d->cfg.ctx_len * 2 * D * act;
            AttnArgs aa{};
            aa.q = ws.qkv; aa.ldq = D; aa.k = kv; aa.v = kv + (size_t)D * act; aa.ldk = 2 * D; aa.out = ws.hbuf; aa.ldo = D;
            aa.q_slot_stride = (size_t)dm.T * D; aa.q_head_stride = dm.d;
            aa.kv_batch_stride = (size_t)d->cfg.ctx_len * 2 * D; aa.kv_head_stride = dm.d;
            aa.Nq = dm.T; aa.Nk = d->cfg.ctx_len; aa.heads = dm.heads; aa.d = dm.d; aa.slots = slots; aa.kv_mod = map.cond_mod;
            {
                ProfScope ps(d, st, DRF_PROF_ATTN, 4.0 * slots * dm.heads * (double)dm.T * d->cfg.ctx_len * dm.d);
                if ((rc = f32 ? launch_attn_f32(aa, st) : launch_attn_bf16(aa, st)) != DRF_OK) return rc;
            }
            if ((rc = gemm(d, ws.hbuf, b.xo, M, epi_resid(ws.resid, D, nullptr, 0, dm.T), st)) != DRF_OK) return rc;
        }
        const bool last = l == n_blocks - 1;
        if ((rc = ln(mrow + 3 * D, mrow + 4 * D, nm, f32 || last)) != DRF_OK) return rc;
        if ((rc = gemm(d, ws.hbuf, b.fc1, M, with_warm(epi_store(ws.mid, dm.R * D, f32, true), f32 ? nullptr : &b.fc2), st, ws.skpart)) != DRF_OK) return rc;
        if (f32 || last) {
            if ((rc = gemm(d, ws.mid, b.fc2, M, epi_resid(ws.resid, D, mrow + 5 * D, nm, dm.T), st, ws.skpart)) != DRF_OK) return rc;
        } else {
            // the attention output may still be pending in ybuf: the MLP output goes to the second buffer
            void* yo = pend1 ? ws.ybuf2 : ws.ybuf;
            if ((rc = gemm(d, ws.mid, b.fc2, M, with_warm(epi_gated(yo, D, mrow + 5 * D, nm, dm.T), &d->blk[l + 1].qkv), st, ws.skpart)) != DRF_OK) return rc;
            (pend1 ? pend2 : pend1) = (const bf16_t*)yo;
        }
    }
    if (resid_out) {
        DRF_HIP(hipMemcpyAsync(resid_out, ws.resid, (size_t)M * D * 4, hipMemcpyDeviceToDevice, st));
        return DRF_OK;
    }
    const float* fm = mod + (size_t)dm.L * 6 * D;           // final shift | scale
    ProfScope ps(d, st, DRF_PROF_ELEMWISE, (double)M * D * 4.0 + (double)M * dm.P * 4.0);
    return launch_final(ws.resid, fm, fm + D, nm, d->fin_w, d->fin_b, dm, slots, eps_out, st);
}

// Algorithmic flops of one slot evaluation: 2 M N K of every Linear of the blocks and of the patch / final
// projections, 4 T^2 D per self-attention (and 4 T ctx_len D per cross-attention), unpadded head width.
double slot_eval_flops(const drf_denoiser* d)
{
    const double D = d->dm.D, T = d->dm.T, R = d->dm.R, P = d->dm.P;
    double per = 2 * T * D * 3 * D + 2 * T * D * D + 2 * 2 * T * D * R * D + 4 * T * T * D;
    if (d->cfg.cond == DRF_COND_TEXT) per += 2 * 2 * T * D * D + 4 * T * (double)d->cfg.ctx_len * D;
    return d->dm.L * per + 2 * 2 * T * D * P;
}

SlotMap identity_map(const int32_t* t)
{
    SlotMap m{};
    m.t_dev = t; m.group = 1; m.x_group = 1; m.x_batch = 1; m.cond_mod = 0;
    return m;
}

// ---- the library's static scratch array ------------------------------------------------------
// drf_eps_batched_static runs the same kernels as drf_eps_batched on buffers carved out of this array
// instead of the handle's workspace, so that the call itself allocates nothing.  Every GPU holds its
// own copy at its own address; in host code the array's name is only a stand-in for the symbol, so the
// device address is looked up once per device (scratch_base) and only that pointer is ever handed to
// kernels.  Nothing in it has to start at zero: every buffer is written by the pass before it is read.
static __device__ __align__(256) unsigned char scratch[DRF_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_base[kMaxDevices] = {};

// Device address of the current device's copy of `scratch`.
drf_status scratch_base(unsigned char** out)
{
    int dev = 0;
    DRF_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) DRF_FAIL(DRF_EUNSUPPORTED, "device index %d beyond the %d the library tracks", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_base[dev]) {
        void* p = nullptr;
        DRF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) DRF_FAIL(DRF_EHIP, "static scratch array has no device address");
        g_scratch_base[dev] = (unsigned char*)p;
    }
    *out = g_scratch_base[dev];
    return DRF_OK;
}

// Lays the Workspace of a `slots`-slot pass out in the static scratch array (256-byte aligned pieces).
drf_status carve_static(const drf_denoiser* d, int slots, Workspace* ws)
{
    unsigned char* base = nullptr;
    drf_status rc = scratch_base(&base);
    if (rc != DRF_OK) return rc;
    const WorkspaceBytes b = workspace_bytes(d, (size_t)slots, (size_t)slots, (size_t)slots);
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = base + off; off += (bytes + 255) / 256 * 256; return p; };
    // bf16: the split-K partial tiles come first, always, so that this entry point splits exactly where
    // drf_eps_batched does and the two return the same bits
    ws->skpart = d->bf16 ? (float*)take(gemm_splitk_scratch_bytes()) : nullptr;
    ws->resid = (float*)take(b.resid); ws->hbuf = take(b.hbuf); ws->qkv = take(b.qkv); ws->mid = take(b.mid);
    ws->ybuf = take(b.ybuf); ws->ybuf2 = take(b.ybuf2);
    ws->mod = (float*)take(b.mod); ws->cact32 = (float*)take(b.cact32); ws->cscratch = (float*)take(b.cscratch); ws->cact = take(b.cact);
    ws->xkv = take(b.xkv); ws->ctx_act = take(b.ctx_act);
    if (off > (size_t)DRF_STATIC_SCRATCH_BYTES)
        DRF_FAIL(DRF_ESHAPE, "a pass of %d slots needs %zu bytes of scratch; the static array holds %zu", slots, off,
                 (size_t)DRF_STATIC_SCRATCH_BYTES);
    return DRF_OK;
}

// ---- one handle in flight -----------------------------------------------------------------------
// Work of two handles (or of the static scratch array's users) overlapping on one GPU from different
// streams is not supported: the kernels are sized for sole occupancy of the chip and the static array
// is shared.  Every enqueueing call first checks that the handle that enqueued last has finished, or
// was used on the same stream (stream order then serialises the two), and records an event behind
// its own work.  Skipped while the stream is being captured (an event recorded there cannot be queried).
std::mutex g_flight_mu;
drf_denoiser* g_last_handle = nullptr;

bool capturing(hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cs != hipStreamCaptureStatusNone;
}

drf_status claim_device(drf_denoiser* d, hipStream_t st)
{
    if (capturing(st)) return DRF_OK;
    std::lock_guard<std::mutex> lk(g_flight_mu);
    drf_denoiser* o = g_last_handle;
    if (o && o->last_stream != st && o->done) {
        // also o == d: the same handle moved to another stream while its buffers are still in use
        const hipError_t q = hipEventQuery(o->done);
        if (q == hipErrorNotReady) {
            if (o == d) DRF_FAIL(DRF_EUNSUPPORTED, "this handle still has work in flight on another stream; synchronise that stream first");
            DRF_FAIL(DRF_EUNSUPPORTED, "another denoiser handle still has work in flight on a different stream; "
                                       "synchronise that stream first (one handle in flight per process)");
        }
        if (q != hipSuccess) (void)hipGetLastError();
    }
    return DRF_OK;
}

drf_status mark_in_flight(drf_denoiser* d, hipStream_t st)
{
    if (capturing(st)) return DRF_OK;
    std::lock_guard<std::mutex> lk(g_flight_mu);
    if (d->done) DRF_HIP(hipEventRecord(d->done, st));
    d->last_stream = st;
    g_last_handle = d;
    return DRF_OK;
}

// An executable graph may still be running on the stream of the handle's last call: wait for that stream
// before the graph's resources go (evictions and mode changes are rare; replays never come here).
void retire_exec(drf_denoiser* d, hipGraphExec_t exec)
{
    if (!exec) return;
    if (hipStreamSynchronize(d->last_stream) != hipSuccess) (void)hipGetLastError();
    (void)hipGraphExecDestroy(exec);
}

void drop_graphs(drf_denoiser* d)
{
    for (GraphEntry& g : d->graphs) retire_exec(d, g.exec);
    d->graphs.clear();
}

bool same_key(const SampleKey& a, const SampleKey& b)
{
    return a.sched.train_steps == b.sched.train_steps && a.sched.beta_start == b.sched.beta_start &&
           a.sched.beta_end == b.sched.beta_end && a.sched.steps == b.sched.steps && a.sched.eta == b.sched.eta &&
           a.sched.sampler == b.sched.sampler && a.sched.shift == b.sched.shift && a.mode == b.mode && a.n == b.n &&
           a.batch == b.batch && a.x_T == b.x_T && a.cond == b.cond && a.null_cond == b.null_cond && a.x_0 == b.x_0 &&
           a.z == b.z && a.cfg_scale == b.cfg_scale && a.has_noise == b.has_noise && a.seed == b.seed &&
           a.field0 == b.field0 && a.ws_gen == b.ws_gen;
}

// The executable graph for a drf_sample call with arguments `key`, or *exec = NULL when this call is to
// run eagerly (first sight of the key in mode 1, or a capture that failed).  The launch sequence is
// captured on a stream of the handle's own (the caller's may be the legacy default stream, which cannot
// be captured), in thread-local mode, and holds kernel nodes only: no memset, no memcpy.
template <typename F> drf_status graph_for_call(drf_denoiser* d, const SampleKey& key, F&& enqueue, hipGraphExec_t* exec)
{
    *exec = nullptr;
    GraphEntry* e = nullptr;
    for (GraphEntry& g : d->graphs)
        if (same_key(g.key, key)) { e = &g; break; }
    if (!e) {
        // entries for buffers that no longer exist go first, then the least recently used
        for (size_t i = 0; i < d->graphs.size();)
            if (d->graphs[i].key.ws_gen != d->ws_gen) {
                retire_exec(d, d->graphs[i].exec);
                d->graphs.erase(d->graphs.begin() + (long)i);
            } else ++i;
        if (d->graphs.size() >= kMaxGraphs) {
            size_t lru = 0;
            for (size_t i = 1; i < d->graphs.size(); ++i)
                if (d->graphs[i].last_use < d->graphs[lru].last_use) lru = i;
            retire_exec(d, d->graphs[lru].exec);
            d->graphs.erase(d->graphs.begin() + (long)lru);
        }
        GraphEntry ne; ne.key = key; ne.last_use = ++d->graph_clock;
        d->graphs.push_back(ne);
        if (d->graph_mode != 2) return DRF_OK;      // first sight: eager
        e = &d->graphs.back();
    }
    e->last_use = ++d->graph_clock;
    if (e->failed) return DRF_OK;
    if (!e->exec) {
        if (!d->cap_stream) DRF_HIP(hipStreamCreateWithFlags(&d->cap_stream, hipStreamNonBlocking));
        DRF_HIP(hipStreamBeginCapture(d->cap_stream, hipStreamCaptureModeThreadLocal));
        const drf_status rc = enqueue(d->cap_stream);
        hipGraph_t graph = nullptr;
        const hipError_t ee = hipStreamEndCapture(d->cap_stream, &graph);
        hipGraphExec_t ex = nullptr;
        if (rc == DRF_OK && ee == hipSuccess && graph && hipGraphInstantiate(&ex, graph, nullptr, nullptr, 0) == hipSuccess) {
            e->exec = ex;
        } else {
            (void)hipGetLastError();
            e->failed = true;                       // this key runs eagerly from now on
        }
        if (graph) (void)hipGraphDestroy(graph);
        if (rc != DRF_OK) return rc;
    }
    *exec = e->exec;
    return DRF_OK;
}

drf_status eps_common(drf_denoiser* den, const float* x, const int32_t* t, const void* cond, int slots, int n_blocks,
                      float* eps_out, float* resid_out, hipStream_t st, bool static_scratch = false)
{
    if (!den) DRF_FAIL(DRF_EINVAL, "denoiser is NULL");
    if (slots < 0) DRF_FAIL(DRF_EINVAL, "slots must be >= 0");
    if (slots == 0) return DRF_OK;
    if (!x || !t || !cond || (!eps_out && !resid_out)) DRF_FAIL(DRF_EINVAL, "NULL buffer");
    if ((size_t)slots * den->dm.T > (size_t)1 << 30) DRF_FAIL(DRF_EINVAL, "slots * tokens too large");
    if (slots > kMaxSlots) DRF_FAIL(DRF_ESHAPE, "a pass of %d slots exceeds the %d the launches cover", slots, kMaxSlots);
    drf_status rc;
    if ((rc = claim_device(den, st)) != DRF_OK) return rc;
    Workspace ws;
    if (static_scratch) {
        if ((rc = carve_static(den, slots, &ws)) != DRF_OK) return rc;
    } else {
        if ((rc = ensure_workspace(den, slots, st)) != DRF_OK) return rc;
        if ((rc = ensure_cond(den, slots, st)) != DRF_OK) return rc;
        if ((rc = ensure_ctx(den, slots, st)) != DRF_OK) return rc;
        ws = den->ws;
    }
    if (den->cfg.cond == DRF_COND_TEXT && (rc = compute_ctx_kv(den, ws, (const float*)cond, slots, st)) != DRF_OK) return rc;
    const SlotMap map = identity_map(t);
    if ((rc = conditioning(den, ws, map, cond, slots, 0, ws.mod, st)) != DRF_OK) return rc;
    if ((rc = forward(den, ws, x, map, ws.mod, slots, n_blocks, eps_out, resid_out, st)) != DRF_OK) return rc;
    return mark_in_flight(den, st);
}

}  // namespace

extern "C" size_t drf_denoiser_weight_count(const drf_dit_config* cfg)
{
    if (check_config(cfg) != DRF_OK) return 0;
    return weight_count(cfg);
}

extern "C" drf_status drf_denoiser_create(const drf_dit_config* cfg, const float* host_weights, size_t count,
                                          void* hip_stream, drf_denoiser** out)
{
    drf_status rc = check_config(cfg);
    if (rc != DRF_OK) return rc;
    if (!host_weights || !out) DRF_FAIL(DRF_EINVAL, "NULL argument");
    *out = nullptr;
    const size_t want = weight_count(cfg);
    if (count != want) DRF_FAIL(DRF_EINVAL, "weight count %zu does not match configuration (%zu)", count, want);
    hipStream_t st = (hipStream_t)hip_stream;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { (void)hipGetLastError(); DRF_FAIL(DRF_EHIP, "no HIP device available"); }

    drf_denoiser* d = new (std::nothrow) drf_denoiser();
    if (!d) DRF_FAIL(DRF_ENOMEM, "host allocation failed");
    d->cfg = *cfg;
    d->bf16 = cfg->dtype == DRF_BF16;
    DitDims& dm = d->dm;
    dm.D = cfg->hidden; dm.P = cfg->in_ch * cfg->patch * cfg->patch; dm.gh = cfg->lat_h / cfg->patch; dm.gw = cfg->lat_w / cfg->patch;
    dm.T = dm.gh * dm.gw; dm.C = cfg->in_ch; dm.H = cfg->lat_h; dm.W = cfg->lat_w; dm.patch = cfg->patch; dm.heads = cfg->heads;
    dm.d = cfg->hidden / cfg->heads; dm.R = cfg->mlp_ratio; dm.L = cfg->depth;
    d->n_mod = 6 * dm.L * dm.D + 2 * dm.D;
    const size_t D = (size_t)dm.D, P = (size_t)dm.P, R = (size_t)dm.R;

    auto fail = [&](drf_status s) { drf_denoiser_destroy(d); return s; };

    // In bf16 mode every parameter takes its bf16 value first (round-to-nearest-even).
    std::vector<float> rounded;
    const float* src = host_weights;
    if (d->bf16) {
        rounded.resize(count);
        for (size_t i = 0; i < count; ++i) rounded[i] = rne_bf16(host_weights[i]);
        src = rounded.data();
    }
    if ((rc = dev_alloc(d, (void**)&d->params32, count * 4)) != DRF_OK) return fail(rc);
    if (hipMemcpy(d->params32, src, count * 4, hipMemcpyHostToDevice) != hipSuccess) { set_error("weight upload failed"); return fail(DRF_EHIP); }

    // Walk the documented order; collect matrices that the GEMMs use.
    size_t off = 0;
    auto take = [&](size_t n) { const float* p = d->params32 + off; off += n; return p; };
    struct Pending { LinearW* lw; size_t woff; };
    std::vector<Pending> mats;
    auto take_linear = [&](LinearW* lw, size_t N, size_t K) {
        mats.push_back({ lw, off });
        lw->w32 = take(N * K); lw->b = take(N); lw->N = (int)N; lw->K = (int)K;
    };
    d->patch_w = take(D * P); d->patch_b = take(D);
    d->t_w1 = take(D * kTFreq); d->t_b1 = take(D); d->t_w2 = take(D * D); d->t_b2 = take(D);
    if (cfg->cond == DRF_COND_VECTOR) { d->c_w = take(D * (size_t)cfg->cond_dim); d->c_b = take(D); }
    else if (cfg->cond == DRF_COND_CLASS) d->table = take(((size_t)cfg->cond_dim + 1) * D);
    d->blk.resize((size_t)dm.L);
    std::vector<size_t> ada_w_off((size_t)dm.L + 1), ada_b_off((size_t)dm.L + 1);
    for (int l = 0; l < dm.L; ++l) {
        BlockW& b = d->blk[(size_t)l];
        ada_w_off[(size_t)l] = off; take(6 * D * D); ada_b_off[(size_t)l] = off; take(6 * D);
        take_linear(&b.qkv, 3 * D, D);
        take_linear(&b.proj, D, D);
        if (cfg->cond == DRF_COND_TEXT) {
            take_linear(&b.xq, D, D);
            take_linear(&b.xkv, 2 * D, (size_t)cfg->cond_dim);
            take_linear(&b.xo, D, D);
        }
        take_linear(&b.fc1, R * D, D);
        take_linear(&b.fc2, D, R * D);
    }
    ada_w_off[(size_t)dm.L] = off; take(2 * D * D); ada_b_off[(size_t)dm.L] = off; take(2 * D);
    d->fin_w = take(P * D); d->fin_b = take(P);
    if (off != count) { set_error("internal: parameter walk mismatch"); return fail(DRF_EINVAL); }

    // Stack the adaLN projections of all blocks and of the final layer into one [n_mod][D] matrix.
    float *ada_w = nullptr, *ada_b = nullptr;
    if ((rc = dev_alloc(d, (void**)&ada_w, (size_t)d->n_mod * D * 4)) != DRF_OK) return fail(rc);
    if ((rc = dev_alloc(d, (void**)&ada_b, (size_t)d->n_mod * 4)) != DRF_OK) return fail(rc);
    for (int l = 0; l <= dm.L; ++l) {
        const size_t rows = (l < dm.L ? 6 : 2) * D, r0 = (size_t)l * 6 * D;
        if (hipMemcpy(ada_w + r0 * D, d->params32 + ada_w_off[(size_t)l], rows * D * 4, hipMemcpyDeviceToDevice) != hipSuccess ||
            hipMemcpy(ada_b + r0, d->params32 + ada_b_off[(size_t)l], rows * 4, hipMemcpyDeviceToDevice) != hipSuccess) {
            set_error("adaLN repack failed");
            return fail(DRF_EHIP);
        }
    }
    d->ada.w32 = ada_w; d->ada.b = ada_b; d->ada.N = d->n_mod; d->ada.K = dm.D;
    mats.push_back({ &d->ada, (size_t)-1 });

    if (hipDeviceSynchronize() != hipSuccess) { set_error("create: device synchronise failed"); return fail(DRF_EHIP); }
    if (d->bf16) {
        for (Pending& pm : mats) {
            const size_t n = (size_t)pm.lw->N * pm.lw->K;
            bf16_t* w16 = nullptr;
            if ((rc = dev_alloc(d, (void**)&w16, n * 2)) != DRF_OK) return fail(rc);
            if ((rc = launch_f32_to_bf16(pm.lw->w32, w16, n, st)) != DRF_OK) return fail(rc);   // exact: values are bf16 already
            pm.lw->w16 = w16;
        }
    }

    // fixed 2-D sin-cos position code
    {
        std::vector<float> pos((size_t)dm.T * D);
        const size_t q4 = D / 4;
        for (int py = 0; py < dm.gh; ++py)
            for (int px = 0; px < dm.gw; ++px) {
                float* row = pos.data() + ((size_t)py * dm.gw + px) * D;
                for (size_t i = 0; i < q4; ++i) {
                    const double om = std::exp(-std::log(10000.0) * (double)i / (double)q4);
                    row[i] = (float)std::sin(py * om); row[q4 + i] = (float)std::cos(py * om);
                    row[2 * q4 + i] = (float)std::sin(px * om); row[3 * q4 + i] = (float)std::cos(px * om);
                }
            }
        if ((rc = dev_alloc(d, (void**)&d->pos, pos.size() * 4)) != DRF_OK) return fail(rc);
        if (hipMemcpy(d->pos, pos.data(), pos.size() * 4, hipMemcpyHostToDevice) != hipSuccess) { set_error("position code upload failed"); return fail(DRF_EHIP); }
    }
    if (hipStreamSynchronize(st) != hipSuccess) { set_error("create: stream synchronise failed"); return fail(DRF_EHIP); }
    if (d->bf16) {
        // the fp32 copies of the big matrices are no longer needed; keep params32 (small tensors point into it)
        dev_free(d, &ada_w);
        d->ada.w32 = nullptr;
    }
    if (hipEventCreateWithFlags(&d->done, hipEventDisableTiming) != hipSuccess) { set_error("create: event creation failed"); return fail(DRF_EHIP); }
    // the set-up call of the library on this device: look up the device's copy of the static scratch array
    {
        unsigned char* base = nullptr;
        if ((rc = scratch_base(&base)) != DRF_OK) return fail(rc);
    }
    *out = d;
    return DRF_OK;
}

extern "C" void drf_denoiser_destroy(drf_denoiser* den)
{
    if (!den) return;
    {
        std::lock_guard<std::mutex> lk(g_flight_mu);
        if (g_last_handle == den) {
            // its work may still be running: hipFree below waits for the device, after which no other handle can collide with it
            g_last_handle = nullptr;
        }
    }
    drop_graphs(den);
    if (den->cap_stream) (void)hipStreamDestroy(den->cap_stream);
    for (void* p : den->allocs) (void)hipFree(p);
    if (den->done) (void)hipEventDestroy(den->done);
    for (hipEvent_t ev : den->prof.pool) (void)hipEventDestroy(ev);
    delete den;
}

extern "C" drf_status drf_denoiser_reserve(drf_denoiser* den, int max_slots)
{
    if (!den || max_slots < 0) DRF_FAIL(DRF_EINVAL, "bad argument");
    drf_status rc = ensure_workspace(den, max_slots, den->last_stream);
    if (rc == DRF_OK) rc = ensure_cond(den, max_slots, den->last_stream);
    return rc != DRF_OK ? rc : ensure_ctx(den, max_slots, den->last_stream);
}

extern "C" drf_status drf_eps_batched(drf_denoiser* den, const float* x, const int32_t* t, const void* cond, int slots,
                                      float* eps_out, void* hip_stream)
{
    if (slots > 0 && !eps_out) DRF_FAIL(DRF_EINVAL, "eps_out is NULL");
    return eps_common(den, x, t, cond, slots, den ? den->dm.L : 0, eps_out, nullptr, (hipStream_t)hip_stream);
}

extern "C" drf_status drf_eps_batched_static(drf_denoiser* den, const float* x, const int32_t* t, const void* cond,
                                             int slots, float* eps_out, void* hip_stream)
{
    if (slots > 0 && !eps_out) DRF_FAIL(DRF_EINVAL, "eps_out is NULL");
    if (den && den->prof.on) DRF_FAIL(DRF_EUNSUPPORTED, "per-launch profiling creates events; switch it off for the no-allocation call");
    return eps_common(den, x, t, cond, slots, den ? den->dm.L : 0, eps_out, nullptr, (hipStream_t)hip_stream, true);
}

extern "C" drf_status drf_eps_trace(drf_denoiser* den, const float* x, const int32_t* t, const void* cond, int slots,
                                    int n_blocks, float* resid_out, void* hip_stream)
{
    if (!den) DRF_FAIL(DRF_EINVAL, "denoiser is NULL");
    if (n_blocks < 0 || n_blocks > den->dm.L) DRF_FAIL(DRF_EINVAL, "n_blocks %d outside [0, %d]", n_blocks, den->dm.L);
    if (slots > 0 && !resid_out) DRF_FAIL(DRF_EINVAL, "resid_out is NULL");
    return eps_common(den, x, t, cond, slots, n_blocks, nullptr, resid_out, (hipStream_t)hip_stream);
}

extern "C" drf_status drf_sample(drf_denoiser* den, const drf_sched_config* sched, drf_mode mode, int n, int batch,
                                 const float* x_T, const void* cond, const void* null_cond, float cfg_scale,
                                 float* x_0_out, void* hip_stream)
{
    return drf_sample_noise(den, sched, mode, n, batch, x_T, cond, null_cond, cfg_scale, nullptr, x_0_out, hip_stream);
}

extern "C" drf_status drf_sample_noise(drf_denoiser* den, const drf_sched_config* sched, drf_mode mode, int n, int batch,
                                       const float* x_T, const void* cond, const void* null_cond, float cfg_scale,
                                       const drf_noise* noise, float* x_0_out, void* hip_stream)
{
    if (!den) DRF_FAIL(DRF_EINVAL, "denoiser is NULL");
    Schedule sch;
    drf_status rc = make_schedule(sched, &sch);
    if (rc != DRF_OK) return rc;
    if (batch < 0) DRF_FAIL(DRF_EINVAL, "batch must be >= 0");
    if (n < 1) DRF_FAIL(DRF_EINVAL, "block size n must be >= 1 (got %d)", n);
    if (n > sch.steps) n = sch.steps;               // larger blocks are cut at index 0 anyway
    if (n > kMaxBlock) DRF_FAIL(DRF_EUNSUPPORTED, "block size n = %d exceeds the built maximum %d", n, kMaxBlock);
    std::vector<Pass> passes;
    if ((rc = build_plan(sch, mode, n, &passes, nullptr)) != DRF_OK) return rc;
    if (batch == 0) return DRF_OK;
    if (!x_T || !cond || !x_0_out) DRF_FAIL(DRF_EINVAL, "NULL buffer");
    // coefficients (and the noise source) of every pass's update, checked before any launch
    std::vector<UpdateArgs> updates(passes.size());
    for (size_t k = 0; k < passes.size(); ++k) {
        const Pass& p = passes[k];
        UpdateArgs& u = updates[k];
        u = UpdateArgs{};
        u.n_chain = (int)p.chain.size();
        for (int i = 0; i < u.n_chain; ++i) {
            if ((rc = sch.coef(p.chain[(size_t)i].first, p.chain[(size_t)i].second, &u.cA[i], &u.cB[i], &u.cC[i])) != DRF_OK) return rc;
            u.cz[i] = p.chain_z[(size_t)i];
        }
        u.n_draft = (int)p.draft_to.size();
        for (int j = 0; j < u.n_draft; ++j) {
            if ((rc = sch.coef(p.s_after, p.draft_to[(size_t)j], &u.dA[j], &u.dB[j], &u.dC[j])) != DRF_OK) return rc;
            u.dz[j] = p.draft_z[(size_t)j];
        }
        if ((rc = set_noise_source(&u, noise)) != DRF_OK) return rc;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const DitDims& dm = den->dm;
    const int g = null_cond ? 2 : 1, gB = g * batch;
    const size_t E = (size_t)dm.C * dm.H * dm.W, field = (size_t)batch * E;
    if ((size_t)n * gB * dm.T > (size_t)1 << 30) DRF_FAIL(DRF_EINVAL, "n * batch * tokens too large");
    if ((size_t)n * gB > kMaxSlots) DRF_FAIL(DRF_ESHAPE, "a pass of %zu slots exceeds the %d the launches cover", (size_t)n * gB, kMaxSlots);

    // buffers: drafts [n][B][E], noises [n][g][B][E], anchor [B][E], conditioning rows [g*B]
    if ((rc = claim_device(den, st)) != DRF_OK) return rc;
    if (n > den->cap_sample_n || den->cap_sample_field < field || g > den->cap_sample_g) {
        DRF_HIP(hipStreamSynchronize(st));
        den->cap_sample_n = 0; den->cap_sample_field = 0; den->cap_sample_g = 0;
        ++den->ws_gen;
        dev_free(den, &den->drafts); dev_free(den, &den->epsbuf); dev_free(den, &den->anchor);
        if ((rc = dev_alloc(den, (void**)&den->drafts, (size_t)n * field * 4)) != DRF_OK) return rc;
        if ((rc = dev_alloc(den, (void**)&den->epsbuf, (size_t)n * g * field * 4)) != DRF_OK) return rc;
        if ((rc = dev_alloc(den, (void**)&den->anchor, field * 4)) != DRF_OK) return rc;
        den->cap_sample_n = n; den->cap_sample_field = field; den->cap_sample_g = g;
    }
    size_t crow = 0;
    switch (den->cfg.cond) {
    case DRF_COND_VECTOR: crow = (size_t)den->cfg.cond_dim * 4; break;
    case DRF_COND_CLASS: crow = 4; break;
    default: crow = (size_t)den->cfg.ctx_len * den->cfg.cond_dim * 4; break;
    }
    if (den->cond_cat_bytes < crow * gB) {
        DRF_HIP(hipStreamSynchronize(st));
        den->cond_cat_bytes = 0;
        ++den->ws_gen;
        dev_free(den, &den->cond_cat);
        if ((rc = dev_alloc(den, &den->cond_cat, crow * gB)) != DRF_OK) return rc;
        den->cond_cat_bytes = crow * gB;
    }
    if ((rc = ensure_workspace(den, n * gB, st)) != DRF_OK) return rc;
    if ((rc = ensure_ctx(den, gB, st)) != DRF_OK) return rc;
    // The conditioning of the passes is known up front (timesteps from the plan, per-sample cond rows): the
    // modulation rows of many passes are produced by a few large launches instead of one small,
    // weight-bandwidth-bound GEMM per pass.  The table holds the rows of a chunk of consecutive passes
    // (at least one pass, otherwise up to kCondChunkRows rows), so its size does not grow with the
    // number of sampling steps times the batch.
    size_t max_pass_rows = 0;
    for (const Pass& p : passes) max_pass_rows = std::max(max_pass_rows, p.eval_s.size() * (size_t)gB);
    const size_t table_rows = std::max(max_pass_rows, (size_t)kCondChunkRows);
    if ((rc = ensure_cond(den, (int)table_rows, st)) != DRF_OK) return rc;

    // the caller's conditioning rows, cond then null: copied eagerly (also ahead of a graph replay)
    DRF_HIP(hipMemcpyAsync(den->cond_cat, cond, crow * batch, hipMemcpyDeviceToDevice, st));
    if (g == 2) DRF_HIP(hipMemcpyAsync((char*)den->cond_cat + crow * batch, null_cond, crow * batch, hipMemcpyDeviceToDevice, st));

    // Everything after this point is a fixed sequence of kernel launches whose arguments depend only on
    // the call's arguments and the handle's buffers.
    const Workspace& ws = den->ws;
    auto enqueue = [&](hipStream_t es) -> drf_status {
        drf_status r;
        // cross-attention K/V depend only on the context: once per call, for the g*B distinct rows
        if (den->cfg.cond == DRF_COND_TEXT && (r = compute_ctx_kv(den, ws, (const float*)den->cond_cat, gB, es)) != DRF_OK) return r;
        const float* x_anchor = x_T;                // state the next stand-alone pass evaluates
        size_t chunk_end = 0, mod_row = 0;          // passes [.., chunk_end) have their rows in the table; next free row
        for (size_t k = 0; k < passes.size(); ++k) {
            const Pass& p = passes[k];
            const int groups = (int)p.eval_s.size();
            if (k == chunk_end) {
                // conditioning rows of the next chunk of passes, laid out pass after pass from row 0
                SlotMap cmap{};
                cmap.t_dev = nullptr; cmap.group = gB; cmap.x_group = 1; cmap.x_batch = 1; cmap.cond_mod = gB;
                int ng = 0, row0 = 0;
                size_t rows = 0;
                auto flush = [&]() -> drf_status {
                    if (ng == 0) return DRF_OK;
                    drf_status fr = conditioning(den, ws, cmap, den->cond_cat, ng * gB, row0, ws.mod + (size_t)row0 * den->n_mod, es);
                    row0 += ng * gB; ng = 0;
                    return fr;
                };
                while (chunk_end < passes.size() && (rows == 0 || rows + passes[chunk_end].eval_s.size() * gB <= table_rows)) {
                    for (int s_eval : passes[chunk_end].eval_s) {
                        cmap.taus[ng++] = sch.net_time(s_eval);
                        if ((ng == kMaxBlock || (size_t)(ng + 1) * gB > (size_t)kMaxSlots) && (r = flush()) != DRF_OK) return r;
                    }
                    rows += passes[chunk_end].eval_s.size() * gB;
                    ++chunk_end;
                }
                if ((r = flush()) != DRF_OK) return r;
                mod_row = 0;
            }
            SlotMap map{};
            map.t_dev = nullptr; map.group = gB; map.x_group = gB; map.x_batch = batch; map.cond_mod = gB;
            for (int i = 0; i < groups; ++i) map.taus[i] = sch.net_time(p.eval_s[(size_t)i]);
            const float* xin = p.solo ? x_anchor : den->drafts;
            {
                ProfScope pass_scope(den, es, !p.solo && groups == n ? DRF_PROF_PASS_FULL : DRF_PROF_PASS_OTHER,
                                     (double)groups * gB * slot_eval_flops(den));
                if ((r = forward(den, ws, xin, map, ws.mod + mod_row * den->n_mod, groups * gB, dm.L, den->epsbuf, nullptr, es)) != DRF_OK) return r;
            }
            mod_row += (size_t)groups * gB;

            UpdateArgs& u = updates[k];
            u.x_base = p.base_is_draft ? den->drafts : x_anchor;
            u.eps = den->epsbuf; u.field = field; u.g = g; u.w = cfg_scale;
            u.anchor_field = p.anchor_field < 0 ? 0 : p.anchor_field;
            if (p.writes_x0) {
                if (u.n_draft > 0) { u.draft_out = x_0_out; u.x_out = nullptr; }      // the lone draft to index 0 is x_0
                else { u.x_out = x_0_out; u.draft_out = nullptr; }
            } else if (u.n_draft > 0) {
                // drafts overwrite the buffer the chain started from: each element is read before it is written
                u.draft_out = den->drafts; u.x_out = nullptr;
            } else {
                u.x_out = den->anchor; u.draft_out = nullptr;
                x_anchor = den->anchor;
            }
            const double bytes = (double)field * 4.0 * (1.0 + (double)g * (u.n_chain + (u.n_draft > 0 ? 1 : 0)) + (u.x_out ? 1 : 0) + u.n_draft);
            ProfScope ps(den, es, DRF_PROF_UPDATE, bytes);
            if ((r = launch_update(u, es)) != DRF_OK) return r;
        }
        return DRF_OK;
    };

    // Graph replay: the launch sequence of a call is captured once into a HIP graph and replayed by later
    // calls with the same arguments (same schedule, mode, n, batch, buffers, guidance, noise source), which
    // removes the per-launch host cost that bounds the small configurations.  The first call with a new set
    // of arguments runs eagerly; the second captures.  Not used while profiling or inside a caller's capture.
    SampleKey key{};
    key.sched = *sched; key.mode = mode; key.n = n; key.batch = batch; key.x_T = x_T; key.cond = cond; key.null_cond = null_cond;
    key.cfg_scale = cfg_scale; key.x_0 = x_0_out; key.ws_gen = den->ws_gen;
    if (noise) { key.has_noise = 1; key.z = noise->z; key.seed = noise->seed; key.field0 = noise->field0; }
    if (den->graph_mode != 0 && den->prof.on == 0 && !capturing(st)) {
        hipGraphExec_t exec = nullptr;
        if ((rc = graph_for_call(den, key, enqueue, &exec)) != DRF_OK) return rc;
        if (exec) {
            DRF_HIP(hipGraphLaunch(exec, st));
            ++den->graph_replays;
            return mark_in_flight(den, st);
        }
    }
    if ((rc = enqueue(st)) != DRF_OK) return rc;
    return mark_in_flight(den, st);
}

extern "C" drf_status drf_denoiser_use_graphs(drf_denoiser* den, int mode)
{
    if (!den) DRF_FAIL(DRF_EINVAL, "denoiser is NULL");
    if (mode < 0 || mode > 2) DRF_FAIL(DRF_EINVAL, "graph mode %d outside 0..2", mode);
    den->graph_mode = mode;
    if (mode == 0) drop_graphs(den);
    return DRF_OK;
}

extern "C" drf_status drf_graph_stats(drf_denoiser* den, int* captured, int* failed, long long* replays)
{
    if (!den || !captured || !failed || !replays) DRF_FAIL(DRF_EINVAL, "bad argument");
    *captured = *failed = 0;
    for (const GraphEntry& g : den->graphs) { *captured += g.exec ? 1 : 0; *failed += g.failed ? 1 : 0; }
    *replays = den->graph_replays;
    return DRF_OK;
}

extern "C" drf_status drf_profile_enable(drf_denoiser* den, int on)
{
    if (!den) DRF_FAIL(DRF_EINVAL, "denoiser is NULL");
    if (on < 0 || on > 2) DRF_FAIL(DRF_EINVAL, "profile mode %d outside 0..2", on);
    den->prof.on = on;
    return DRF_OK;
}

extern "C" drf_status drf_profile_read(drf_denoiser* den, int which, long long* launches, double* ms, double* work)
{
    if (!den || !launches || !ms || !work || which < 0 || which >= DRF_PROF_FAMILIES) DRF_FAIL(DRF_EINVAL, "bad argument");
    DRF_HIP(hipDeviceSynchronize());
    Prof& p = den->prof;
    *launches = 0; *ms = 0.0; *work = 0.0;
    std::vector<Prof::Rec> keep;
    for (const Prof::Rec& r : p.recs) {
        if (r.fam != which) { keep.push_back(r); continue; }
        float t = 0.f;
        if (hipEventElapsedTime(&t, p.pool[r.e0], p.pool[r.e1]) == hipSuccess) { *ms += t; *work += r.work; ++*launches; }
        else (void)hipGetLastError();
    }
    p.recs.swap(keep);
    if (p.recs.empty()) p.used = 0;
    return DRF_OK;
}

extern "C" drf_status drf_probe_gemm_bf16(const void* A, const void* W, int M, int N, int K, void* out_bf16,
                                          const float* bias, int variant, void* hip_stream)
{
    if (!A || !W || !out_bf16 || !bias || M < 0 || N < 0 || K < 0) DRF_FAIL(DRF_EINVAL, "bad argument");
    Epilogue e{};
    e.mode = EPI_STORE; e.out = out_bf16; e.ldo = N; e.out_f32 = 0; e.bias = bias;
    // variant 10 (the 128 x 128 tile, K split across workgroups where the rule allows): partial tiles in a buffer
    // that the probe allocates once per process and keeps
    static float* probe_splitk = nullptr;
    if (variant == 10 && !probe_splitk) DRF_HIP(hipMalloc((void**)&probe_splitk, gemm_splitk_scratch_bytes()));
    return launch_gemm_bf16((const bf16_t*)A, (const bf16_t*)W, M, N, K, e, (hipStream_t)hip_stream, variant,
                            variant == 10 ? probe_splitk : nullptr);
}

extern "C" drf_status drf_probe_attn_bf16(const void* qkv, void* out, int slots, int tokens, int heads, int head_dim,
                                          void* hip_stream)
{
    if (!qkv || !out || slots < 0 || tokens < 1 || heads < 1 || head_dim < 1) DRF_FAIL(DRF_EINVAL, "bad argument");
    const int D = heads * head_dim;
    AttnArgs aa{};
    aa.q = qkv; aa.ldq = 3 * D; aa.k = (const bf16_t*)qkv + D; aa.v = (const bf16_t*)qkv + 2 * D; aa.ldk = 3 * D;
    aa.q_slot_stride = aa.kv_batch_stride = (size_t)tokens * 3 * D; aa.q_head_stride = aa.kv_head_stride = head_dim;
    aa.out = out; aa.ldo = D; aa.Nq = tokens; aa.Nk = tokens; aa.heads = heads; aa.d = head_dim; aa.slots = slots; aa.kv_mod = 0;
    return launch_attn_bf16(aa, (hipStream_t)hip_stream);
}
