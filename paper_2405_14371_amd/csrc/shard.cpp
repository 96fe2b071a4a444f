// Shard runtime and C-ABI (see include/shard.h): weight packing, the pre-allocated paged
// KV pool, per-call validation, and the per-layer launch sequence for the prefill and the
// autoregressive phase.  All arithmetic of the layer happens in the kernels; this file
// only moves pointers.
#include "../../include/shard.h"
#include "../../include/shard_introspect.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.hpp"

using namespace shk;

thread_local shk::LaunchTimer shk::g_launch_timer;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(e_ == hipErrorOutOfMemory ? SHARD_E_NOMEM : SHARD_E_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                               \
    } while (0)

struct LayerDev {
    void* wqkv = nullptr;  // [(Hq+2Hkv)*dh, d]   rows: all q heads, all k heads, all v heads
    void* wo = nullptr;    // [d, Hq*dh]
    void* wgu = nullptr;   // [2F, d]             row 2f = gate_f, row 2f+1 = up_f
    void* wd = nullptr;    // [d, F]
    float* g_attn = nullptr;
    float* g_ffn = nullptr;
    void* k = nullptr;     // [n_pages, Hkv, page, dh]
    void* v = nullptr;
};

struct Timing {
    bool on = false;
    std::vector<hipEvent_t> ev[SHARD_K_COUNT];  // start, stop, start, stop, ...
    size_t used[SHARD_K_COUNT] = {0};
    int64_t launches[SHARD_K_COUNT] = {0};
    double seconds[SHARD_K_COUNT] = {0};
    hipStream_t last_stream = nullptr;
};

}  // namespace

// Split-K scratch of the prefill GEMM: slices x M x N floats with slices * tiles <= 512 tiles of
// at most 64 x 128 outputs.
constexpr size_t SPLITK_FLOATS = 512ull * 64 * 128;

struct shard {
    shard_model_cfg m{};
    shard_kv_cfg kv{};
    int layer_lo = 0, layer_hi = 0, L = 0;
    int es = 4;           // bytes per weight / cache element
    int nqkv = 0, nq = 0;
    int max_pages = 0, n_pages = 0, mmax = 0;
    std::vector<LayerDev> layers;
    float2* rope = nullptr;          // [max_seq_len, dh/2]
    int32_t* block_table = nullptr;  // device [max_seqs, max_pages]
    std::vector<int32_t> free_pages; // stack
    std::vector<int32_t> seq_len;    // -1 = slot not live
    std::vector<int32_t> seq_pages;  // pages held per slot
    std::vector<int32_t> host_table; // mirror of block_table
    // Workspaces.  Set 0 holds mmax rows (prefill); the others hold SHARD_MAX_BATCH rows and let
    // decode calls on different streams run side by side.  A set belongs to the stream that
    // used it last; another stream takes it over only after waiting for that use (an event).
    struct Work {
        void* h = nullptr;     // [rows, d]      normalised activations (weight dtype)
        float* q = nullptr;    // [rows, Hq*dh]
        void* o = nullptr;     // [rows, Hq*dh]  attention output (fp32 in decode, weight dtype in prefill)
        void* f = nullptr;     // [rows, F]      SwiGLU output   (same)
        float* part_o = nullptr;
        float* part_ml = nullptr;
        float* splitk = nullptr;   // SPLITK_FLOATS floats
        size_t rows = 0;       // activation rows the set can hold
        hipStream_t owner = nullptr;
        bool used = false;
        uint64_t last_use = 0;
        hipEvent_t done = nullptr;  // recorded after every use
    };
    Work work[SHARD_MAX_STREAMS];
    uint64_t use_clock = 0;
    int nsplit_max = 32;
    Timing timing;
    uint32_t* cvt_flag = nullptr;   // overflow flag of the bf16 -> half conversion during create
    uint32_t* oflow = nullptr;      // host-visible (pinned, mapped) word: a half store left half's range
    void* static_scratch = nullptr; // this device's copy of the library's static scratch array
    std::vector<hipEvent_t> layer_ev;  // L+1 events, used by shard_profile
    bool record_layers = false;
};

namespace {

void free_all(shard* s) {
    for (auto& l : s->layers) {
        void* ptrs[] = {l.wqkv, l.wo, l.wgu, l.wd, l.g_attn, l.g_ffn, l.k, l.v};
        for (void* p : ptrs)
            if (p) (void)hipFree(p);
    }
    void* ptrs[] = {s->rope, s->block_table, s->cvt_flag};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (s->oflow) (void)hipHostFree(s->oflow);
    for (auto& w : s->work) {
        void* wp[] = {w.h, w.q, w.o, w.f, w.part_o, w.part_ml, w.splitk};
        for (void* p : wp)
            if (p) (void)hipFree(p);
        if (w.done) (void)hipEventDestroy(w.done);
    }
    for (auto& v : s->timing.ev)
        for (hipEvent_t e : v) (void)hipEventDestroy(e);
    for (hipEvent_t e : s->layer_ev) (void)hipEventDestroy(e);
    delete s;
}

int validate_cfg(const shard_model_cfg* m, const shard_kv_cfg* kv, int lo, int hi) {
    if (!m || !kv) return fail(SHARD_E_INVAL, "null configuration");
    if (lo < 0 || hi <= lo) return fail(SHARD_E_INVAL, "layer range [%d,%d) is empty or negative", lo, hi);
    if (m->d_model <= 0 || m->n_heads <= 0 || m->n_kv_heads <= 0 || m->ffn_dim <= 0)
        return fail(SHARD_E_INVAL, "model dimensions must be positive");
    if (m->head_dim != 32 && m->head_dim != 64 && m->head_dim != 128)
        return fail(SHARD_E_INVAL, "head_dim %d unsupported (32, 64, 128)", m->head_dim);
    if (m->n_heads % m->n_kv_heads) return fail(SHARD_E_INVAL, "n_heads %% n_kv_heads != 0");
    if (m->d_model % 8 || m->ffn_dim % 8)
        return fail(SHARD_E_INVAL, "d_model and ffn_dim must be multiples of 8 (16-byte rows)");
    if (m->weight_dtype != SHARD_F32 && m->weight_dtype != SHARD_BF16)
        return fail(SHARD_E_INVAL, "unknown weight_dtype %d", m->weight_dtype);
    if (m->act_dtype != SHARD_F32) return fail(SHARD_E_INVAL, "act_dtype must be SHARD_F32");
    if (!(m->rms_eps >= 0.f) || !(m->rope_theta > 0.f)) return fail(SHARD_E_INVAL, "bad rms_eps / rope_theta");
    if (kv->max_seqs < 1 || kv->max_seq_len < 1 || kv->page_size < 1 || kv->max_batch_tokens < 0)
        return fail(SHARD_E_INVAL, "bad KV configuration");
    if (static_cast<uint64_t>(kv->max_seq_len) * static_cast<uint64_t>(kv->page_size) >= (1ull << 32))
        return fail(SHARD_E_INVAL, "max_seq_len * page_size must be below 2^32");
    const uint64_t pages = (static_cast<uint64_t>(kv->max_seq_len) + kv->page_size - 1) / kv->page_size * static_cast<uint64_t>(kv->max_seqs);
    if (pages >= (1ull << 31)) return fail(SHARD_E_INVAL, "max_seqs * ceil(max_seq_len / page_size) must be below 2^31 pages");
    if (static_cast<uint64_t>(m->n_heads) * m->head_dim >= (1ull << 24) || static_cast<uint64_t>(m->d_model) >= (1ull << 24) ||
        static_cast<uint64_t>(m->ffn_dim) >= (1ull << 24))
        return fail(SHARD_E_INVAL, "model widths must be below 2^24");
    return SHARD_OK;
}

// While alive and timing is enabled, every kernel launched on this thread is timed into `klass`.
struct Bracket {
    struct Ctx { shard* s; int klass; hipStream_t st; } ctx;
    static bool next(void* p, hipEvent_t* start, hipEvent_t* stop) {
        Ctx* c = static_cast<Ctx*>(p);
        Timing& t = c->s->timing;
        auto& v = t.ev[c->klass];
        if (t.used[c->klass] + 2 > v.size()) {
            if (v.size() >= (1u << 16)) return false;  // bounded; further launches go untimed
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return false;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return false; }
            v.push_back(a);
            v.push_back(b);
        }
        *start = v[t.used[c->klass]];
        *stop = v[t.used[c->klass] + 1];
        t.used[c->klass] += 2;
        t.last_stream = c->st;
        return true;
    }
    Bracket(shard* s, int klass, hipStream_t st) : ctx{s, klass, st} {
        if (!s->timing.on) return;
        shk::g_launch_timer.next = &Bracket::next;
        shk::g_launch_timer.ctx = &ctx;
    }
    ~Bracket() { shk::g_launch_timer = shk::LaunchTimer{}; }
    Bracket(const Bracket&) = delete;
    Bracket& operator=(const Bracket&) = delete;
};

KvView kv_view(const shard* s, int li) {
    KvView v;
    v.k = s->layers[li].k;
    v.v = s->layers[li].v;
    v.block_table = s->block_table;
    v.max_pages = s->max_pages;
    v.page = s->kv.page_size;
    v.hkv = s->m.n_kv_heads;
    v.dh = s->m.head_dim;
    v.page_magic = v.page >= 2 ? static_cast<uint32_t>(((1ull << 32) + v.page - 1) / v.page) : 0u;
    return v;
}

// Reserve pages so that every sequence of the batch can hold `add` more tokens, and
// enqueue the block-table writes.  Cannot fail: the pool holds max_pages per sequence.
void grow_sequences(shard* s, const SeqBatch& sb, int add, hipStream_t st) {
    TableUpdate u;
    u.n = 0;
    for (int b = 0; b < sb.n; ++b) {
        const int seq = sb.seq[b];
        const int need = (sb.pos[b] + add + s->kv.page_size - 1) / s->kv.page_size;
        while (s->seq_pages[seq] < need) {
            const int32_t page = s->free_pages.back();
            s->free_pages.pop_back();
            const int idx = seq * s->max_pages + s->seq_pages[seq]++;
            s->host_table[idx] = page;
            u.idx[u.n] = idx;
            u.val[u.n] = page;
            if (++u.n == 128) {
                launch_table_update(s->block_table, u, st);
                u.n = 0;
            }
        }
    }
    if (u.n) launch_table_update(s->block_table, u, st);
}

int check_batch(shard* s, const int32_t* seq_ids, int B, int T, bool decode, SeqBatch* sb) {
    if (!s) return fail(SHARD_E_INVAL, "null shard");
    if (!seq_ids) return fail(SHARD_E_INVAL, "null seq_ids");
    if (B < 1 || B > SHARD_MAX_BATCH) return fail(SHARD_E_INVAL, "B=%d outside 1..%d", B, SHARD_MAX_BATCH);
    if (T < 1) return fail(SHARD_E_INVAL, "T=%d < 1", T);
    if (static_cast<long>(B) * T > s->mmax)
        return fail(SHARD_E_INVAL, "B*T=%ld exceeds max_batch_tokens=%d", static_cast<long>(B) * T, s->mmax);
    sb->n = B;
    for (int b = 0; b < B; ++b) {
        const int id = seq_ids[b];
        if (id < 0 || id >= s->kv.max_seqs || s->seq_len[id] < 0)
            return fail(SHARD_E_STATE, "seq_id %d is not live", id);
        for (int c = 0; c < b; ++c)
            if (seq_ids[c] == id) return fail(SHARD_E_STATE, "seq_id %d appears twice in the batch", id);
        if (decode && s->seq_len[id] == 0) return fail(SHARD_E_STATE, "decode on empty sequence %d", id);
        if (s->seq_len[id] + T > s->kv.max_seq_len)
            return fail(SHARD_E_KV_FULL, "sequence %d: %d cached + %d new > max_seq_len %d", id, s->seq_len[id], T,
                        s->kv.max_seq_len);
        sb->seq[b] = id;
        sb->pos[b] = s->seq_len[id];
    }
    return SHARD_OK;
}

void mark_layer(shard* s, int i, hipStream_t st) {
    if (s->record_layers) (void)hipEventRecord(s->layer_ev[i], st);
}

void run_prefill(shard* s, shard::Work& wk, const SeqBatch& sb, int T, const float* x_in, float* x_out, hipStream_t st) {
    const shard_model_cfg& m = s->m;
    const int M = sb.n * T;
    const int dt = m.weight_dtype == SHARD_F32 ? DT_F32 : DT_F16;    // weights as stored on the device
    const int adt = m.weight_dtype == SHARD_F32 ? DT_F32 : DT_F16;   // activations and KV cache
    mark_layer(s, 0, st);
    for (int li = 0; li < s->L; ++li) {
        const LayerDev& l = s->layers[li];
        const float* x = li == 0 ? x_in : x_out;
        {
            Bracket t(s, SHARD_K_PREFILL_NORM, st);
            launch_rmsnorm(x, l.g_attn, m.rms_eps, wk.h, adt, M, m.d_model, st);
        }
        PrefillGemm g{};
        g.M = M; g.dt = dt; g.T = T; g.hq = m.n_heads; g.kv = kv_view(s, li); g.rope = s->rope; g.oflow = s->oflow;
        g.A = wk.h; g.W = l.wqkv; g.N = s->nqkv; g.K = m.d_model; g.epi = EPI_QKV; g.q = wk.q;
        {
            Bracket t(s, SHARD_K_PREFILL_QKV, st);
            launch_prefill_gemm(g, sb, st);
        }
        PrefillAttn at{};
        at.q = wk.q; at.o = wk.o; at.out_dtype = adt; at.B = sb.n; at.T = T; at.hq = m.n_heads;
        at.kv_dtype = adt; at.kv = g.kv;
        {
            Bracket t(s, SHARD_K_PREFILL_ATTN, st);
            launch_prefill_attn(at, sb, st);
        }
        g.A = wk.o; g.W = l.wo; g.N = m.d_model; g.K = s->nq; g.epi = EPI_RESID; g.resid = x; g.out = x_out;
        g.part = wk.splitk; g.part_cap = wk.splitk ? SPLITK_FLOATS : 0;
        {
            Bracket t(s, SHARD_K_PREFILL_O, st);
            launch_prefill_gemm(g, sb, st);
        }
        {
            Bracket t(s, SHARD_K_PREFILL_NORM, st);
            launch_rmsnorm(x_out, l.g_ffn, m.rms_eps, wk.h, adt, M, m.d_model, st);
        }
        g.A = wk.h; g.W = l.wgu; g.N = 2 * m.ffn_dim; g.K = m.d_model; g.epi = EPI_SWIGLU; g.out_act = wk.f;
        {
            Bracket t(s, SHARD_K_PREFILL_GATEUP, st);
            launch_prefill_gemm(g, sb, st);
        }
        g.A = wk.f; g.W = l.wd; g.N = m.d_model; g.K = m.ffn_dim; g.epi = EPI_RESID; g.resid = x_out; g.out = x_out;
        {
            Bracket t(s, SHARD_K_PREFILL_DOWN, st);
            launch_prefill_gemm(g, sb, st);
        }
        mark_layer(s, li + 1, st);
    }
}

// Context slices per workgroup unit (a sequence and the query heads that share its KV head):
// enough slices to put about three workgroups on every compute unit, but never slices
// shorter than one trip of the kernel's token loop (longer slices cost little: the trips of
// a slice are software-pipelined).
int max_context(const SeqBatch& sb) {   // the new token included
    int ctx = 1;
    for (int b = 0; b < sb.n; ++b) ctx = ctx > sb.pos[b] + 1 ? ctx : sb.pos[b] + 1;
    return ctx;
}

int pick_nsplit(const shard* s, const SeqBatch& sb) {
    const int ctx = max_context(sb);
    const int kdt = s->m.weight_dtype == SHARD_F32 ? DT_F32 : DT_F16;
    const int units = sb.n * s->m.n_heads / decode_attn_heads_per_group(kdt, s->m.head_dim, s->m.n_heads, s->m.n_kv_heads);
    if (ctx <= decode_attn_single_pass_ctx(kdt, s->m.head_dim, s->m.n_heads, s->m.n_kv_heads)) return 1;
    const int trip = decode_attn_tokens_per_trip(kdt, s->m.head_dim, s->m.n_heads, s->m.n_kv_heads);
    int n = (ctx + trip - 1) / trip;
    const int target = decode_attn_target_workgroups(kdt, s->m.head_dim, s->m.n_heads, s->m.n_kv_heads);
    const int want = (target + units - 1) / units;
    if (n > want) n = want;
    if (n > s->nsplit_max) n = s->nsplit_max;
    return n < 1 ? 1 : n;
}

// Whether a decode step of B sequences takes the matrix-core projections (run_decode_mfma):
// 16-bit weights, more than 4 sequences, and every inner dimension a multiple of the MFMA
// kernels' 64-element K block; otherwise the streaming kernels carry up to 8 rows per pass.
bool decode_on_matrix_cores(const shard_model_cfg& m, int B) {
    return m.weight_dtype != SHARD_F32 && B > 4 && m.d_model % 64 == 0 && m.ffn_dim % 64 == 0 &&
           (m.n_heads * m.head_dim) % 64 == 0;
}

// Decode step with 16-bit weights and more than 4 sequences: projections on the matrix
// cores, one pass over the weights per group of up to 16 sequences (the streaming kernels'
// vector ALUs fall behind the HBM stream from about 8 rows on).  No RMSNorm launches: the
// gains are part of the 16-bit matrices (folded in at create), each residual epilogue also
// leaves a half copy of its result, and the consuming projection takes the row scale
// rsqrt(mean x^2 + eps) from the activation fragments it loads anyway.
void run_decode_mfma(shard* s, shard::Work& wk, const SeqBatch& all, const float* x_in, float* x_out, hipStream_t st) {
    const shard_model_cfg& m = s->m;
    const int d_model = m.d_model;
    mark_layer(s, 0, st);
    {
        Bracket t(s, SHARD_K_DECODE_QKV, st);
        launch_to_half(x_in, wk.h, static_cast<size_t>(all.n) * d_model, s->oflow, st);
    }
    for (int li = 0; li < s->L; ++li) {
        const LayerDev& l = s->layers[li];
        const KvView kvv = kv_view(s, li);
        for (int b0 = 0; b0 < all.n; b0 += 16) {
            SeqBatch sb;
            sb.n = all.n - b0 < 16 ? all.n - b0 : 16;
            for (int i = 0; i < sb.n; ++i) { sb.seq[i] = all.seq[b0 + i]; sb.pos[i] = all.pos[b0 + i]; }
            const int B = sb.n;
            const float* x = (li == 0 ? x_in : x_out) + static_cast<size_t>(b0) * d_model;
            float* y = x_out + static_cast<size_t>(b0) * d_model;
            void* xh = static_cast<char*>(wk.h) + static_cast<size_t>(b0) * d_model * 2;   // half copy of the residual stream
            DecodeLinear d{};
            d.wt = DT_F16; d.nb = B; d.hq = m.n_heads; d.kv = kvv; d.rope = s->rope; d.eps = m.rms_eps; d.oflow = s->oflow;
            {
                Bracket t(s, SHARD_K_DECODE_QKV, st);
                d.W = l.wqkv; d.N = s->nqkv; d.K = d_model; d.xb = xh; d.norm_xb = 1; d.epi = EPI_QKV; d.q = wk.q;
                launch_decode_linear_mfma(d, sb, st);
            }
            {
                DecodeAttn a{};
                a.q = wk.q; a.o = wk.o; a.o_dtype = DT_F16; a.nb = B; a.hq = m.n_heads; a.kv_dtype = DT_F16; a.kv = kvv;
                a.nsplit = pick_nsplit(s, sb); a.part_o = wk.part_o; a.part_ml = wk.part_ml;
                Bracket t(s, SHARD_K_DECODE_ATTN, st);
                launch_decode_attn(a, sb, st);
            }
            {
                d.W = l.wo; d.N = d_model; d.K = s->nq; d.xb = wk.o; d.norm_xb = 0; d.epi = EPI_RESID; d.resid = x; d.out = y;
                d.out_h = xh;
                Bracket t(s, SHARD_K_DECODE_O, st);
                launch_decode_linear_mfma(d, sb, st);
            }
            {
                Bracket t(s, SHARD_K_DECODE_GATEUP, st);
                d.W = l.wgu; d.N = 2 * m.ffn_dim; d.K = d_model; d.xb = xh; d.norm_xb = 1; d.epi = EPI_SWIGLU; d.out_b = wk.f;
                d.out_h = nullptr;
                launch_decode_linear_mfma(d, sb, st);
            }
            {
                d.W = l.wd; d.N = d_model; d.K = m.ffn_dim; d.xb = wk.f; d.norm_xb = 0; d.epi = EPI_RESID; d.resid = y; d.out = y;
                d.out_h = li + 1 < s->L ? xh : nullptr;
                Bracket t(s, SHARD_K_DECODE_DOWN, st);
                launch_decode_linear_mfma(d, sb, st);
            }
        }
        mark_layer(s, li + 1, st);
    }
}

void run_decode(shard* s, shard::Work& wk, const SeqBatch& sb, const float* x_in, float* x_out, hipStream_t st) {
    const shard_model_cfg& m = s->m;
    const int dt = m.weight_dtype == SHARD_F32 ? DT_F32 : DT_F16;
    const int B = sb.n;
    if (decode_on_matrix_cores(m, B)) {
        run_decode_mfma(s, wk, sb, x_in, x_out, st);
        return;
    }
    float* o = static_cast<float*>(wk.o);
    float* f = static_cast<float*>(wk.f);
    mark_layer(s, 0, st);
    for (int li = 0; li < s->L; ++li) {
        const LayerDev& l = s->layers[li];
        const float* x = li == 0 ? x_in : x_out;
        const KvView kvv = kv_view(s, li);
        // the streaming kernels take up to 8 activation rows per pass over the weights
        for (int b0 = 0; b0 < B; b0 += 8) {
            const int nb = B - b0 < 8 ? B - b0 : 8;
            SeqBatch sub;
            sub.n = nb;
            for (int i = 0; i < nb; ++i) { sub.seq[i] = sb.seq[b0 + i]; sub.pos[i] = sb.pos[b0 + i]; }
            DecodeLinear d{};
            d.W = l.wqkv; d.N = s->nqkv; d.K = m.d_model; d.wt = dt; d.nb = nb;
            d.x = x + static_cast<size_t>(b0) * m.d_model; d.gain = l.g_attn; d.eps = m.rms_eps;
            d.epi = EPI_QKV; d.q = wk.q + static_cast<size_t>(b0) * s->nq; d.hq = m.n_heads; d.kv = kvv; d.rope = s->rope;
            d.oflow = s->oflow;
            Bracket t(s, SHARD_K_DECODE_QKV, st);
            launch_decode_linear(d, sub, st);
        }
        {
            DecodeAttn a{};
            a.q = wk.q; a.o = o; a.o_dtype = DT_F32; a.nb = B; a.hq = m.n_heads;
            a.kv_dtype = dt; a.kv = kvv;
            a.nsplit = pick_nsplit(s, sb); a.part_o = wk.part_o; a.part_ml = wk.part_ml;
            Bracket t(s, SHARD_K_DECODE_ATTN, st);
            launch_decode_attn(a, sb, st);
        }
        for (int b0 = 0; b0 < B; b0 += 8) {
            const int nb = B - b0 < 8 ? B - b0 : 8;
            DecodeLinear d{};
            d.W = l.wo; d.N = m.d_model; d.K = s->nq; d.wt = dt; d.nb = nb;
            d.x = o + static_cast<size_t>(b0) * s->nq; d.epi = EPI_RESID; d.oflow = s->oflow;
            d.resid = x + static_cast<size_t>(b0) * m.d_model; d.out = x_out + static_cast<size_t>(b0) * m.d_model;
            Bracket t(s, SHARD_K_DECODE_O, st);
            launch_decode_linear(d, sb, st);
        }
        for (int b0 = 0; b0 < B; b0 += 8) {
            const int nb = B - b0 < 8 ? B - b0 : 8;
            DecodeLinear d{};
            d.W = l.wgu; d.N = 2 * m.ffn_dim; d.K = m.d_model; d.wt = dt; d.nb = nb;
            d.x = x_out + static_cast<size_t>(b0) * m.d_model; d.gain = l.g_ffn; d.eps = m.rms_eps;
            d.epi = EPI_SWIGLU; d.out = f + static_cast<size_t>(b0) * m.ffn_dim; d.oflow = s->oflow;
            Bracket t(s, SHARD_K_DECODE_GATEUP, st);
            launch_decode_linear(d, sb, st);
        }
        for (int b0 = 0; b0 < B; b0 += 8) {
            const int nb = B - b0 < 8 ? B - b0 : 8;
            DecodeLinear d{};
            d.W = l.wd; d.N = m.d_model; d.K = m.ffn_dim; d.wt = dt; d.nb = nb;
            d.x = f + static_cast<size_t>(b0) * m.ffn_dim; d.epi = EPI_RESID; d.oflow = s->oflow;
            d.resid = x_out + static_cast<size_t>(b0) * m.d_model; d.out = x_out + static_cast<size_t>(b0) * m.d_model;
            Bracket t(s, SHARD_K_DECODE_DOWN, st);
            launch_decode_linear(d, sb, st);
        }
        mark_layer(s, li + 1, st);
    }
}

// The workspace set a call with `rows` activation rows on stream `st` uses: a set the stream
// already owns, else a free one (small sets first for small calls, so that the large ones stay
// available to prefill), else the least recently used one that is large enough.  Taking over
// another stream's set first makes `st` wait for that stream's last use of it.
int acquire_work(shard* s, hipStream_t st, size_t rows, shard::Work** out) {
    shard::Work* w = nullptr;
    for (auto& c : s->work)
        if (c.used && c.owner == st && c.rows >= rows) { w = &c; break; }
    for (int i = SHARD_MAX_STREAMS - 1; !w && i >= 0; --i)   // sets are sized large first: search from the back
        if (!s->work[i].used && s->work[i].rows >= rows) w = &s->work[i];
    if (!w) {
        for (auto& c : s->work)
            if (c.rows >= rows && (!w || c.last_use < w->last_use)) w = &c;
    }
    if (!w) return fail(SHARD_E_INVAL, "no workspace holds %zu rows", rows);  // cannot happen: set 0 holds mmax
    if (w->used && w->owner != st) HIP_TRY(hipStreamWaitEvent(st, w->done, 0));
    w->owner = st;
    w->used = true;
    w->last_use = ++s->use_clock;
    *out = w;
    return SHARD_OK;
}

int release_work(shard::Work* w, hipStream_t st) {
    HIP_TRY(hipEventRecord(w->done, st));
    return SHARD_OK;
}

int check_launch() {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SHARD_E_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    const hipError_t a = shk::kernel_attribute_error();
    if (a != hipSuccess)
        return fail(SHARD_E_HIP, "opting a kernel into more than 64 KB of LDS failed: %s", hipGetErrorString(a));
    return SHARD_OK;
}

// Undo of grow_sequences for a call that failed after it: the pages go back on the stack in
// the order they came off (the block-table entries a failed call wrote are beyond seq_pages
// and therefore unused).
struct GrowUndo {
    shard* s;
    int n;
    int32_t seq[SHARD_MAX_BATCH], pages[SHARD_MAX_BATCH];
    GrowUndo(shard* sh, const SeqBatch& sb) : s(sh), n(sb.n) {
        for (int b = 0; b < n; ++b) { seq[b] = sb.seq[b]; pages[b] = sh->seq_pages[sb.seq[b]]; }
    }
    void rollback() {
        for (int b = n - 1; b >= 0; --b)
            while (s->seq_pages[seq[b]] > pages[b]) {
                const int idx = seq[b] * s->max_pages + --s->seq_pages[seq[b]];
                s->free_pages.push_back(s->host_table[idx]);
            }
    }
};

int range_check(const shard* s) {
    if (s->oflow && *static_cast<volatile uint32_t*>(s->oflow))
        return fail(SHARD_E_RANGE, "an activation or KV-cache value left the range of IEEE half (65504) in an earlier call; "
                                   "see shard_overflow");
    return SHARD_OK;
}

// Bytes of the static scratch array a decode step of this batch needs, and the carve-up.
constexpr size_t SCRATCH_ALIGN = 256;
size_t align_up(size_t v) { return (v + SCRATCH_ALIGN - 1) / SCRATCH_ALIGN * SCRATCH_ALIGN; }

// Largest number of context slices any attention launch of this decode step uses (the launch
// sequence of run_decode / run_decode_mfma decides the sub-batches).
int max_nsplit_of_step(const shard* s, const SeqBatch& all) {
    if (!decode_on_matrix_cores(s->m, all.n)) return pick_nsplit(s, all);
    int worst = 1;
    for (int b0 = 0; b0 < all.n; b0 += 16) {
        SeqBatch sb;
        sb.n = all.n - b0 < 16 ? all.n - b0 : 16;
        for (int i = 0; i < sb.n; ++i) { sb.seq[i] = all.seq[b0 + i]; sb.pos[i] = all.pos[b0 + i]; }
        const int n = pick_nsplit(s, sb);
        worst = worst > n ? worst : n;
    }
    return worst;
}

int carve_static(const shard* s, const SeqBatch& sb, shard::Work* w) {
    const size_t B = sb.n, d = s->m.d_model, nq = s->nq, F = s->m.ffn_dim, dh = s->m.head_dim;
    const size_t nsplit = max_nsplit_of_step(s, sb);
    const size_t units = B * s->m.n_heads;
    const size_t sizes[6] = {B * d * sizeof(float), B * nq * sizeof(float), B * nq * sizeof(float), B * F * sizeof(float),
                             units * nsplit * dh * sizeof(float), units * nsplit * 2 * sizeof(float)};
    size_t off[6], total = 0;
    for (int i = 0; i < 6; ++i) { off[i] = total; total += align_up(sizes[i]); }
    if (total > SHARD_STATIC_SCRATCH_BYTES)
        return fail(SHARD_E_INVAL, "this decode step needs %zu bytes of scratch; shard_decode_static has %u (use shard_decode)",
                    total, SHARD_STATIC_SCRATCH_BYTES);
    char* base = static_cast<char*>(s->static_scratch);
    w->h = base + off[0];
    w->q = reinterpret_cast<float*>(base + off[1]);
    w->o = base + off[2];
    w->f = base + off[3];
    w->part_o = reinterpret_cast<float*>(base + off[4]);
    w->part_ml = reinterpret_cast<float*>(base + off[5]);
    w->splitk = nullptr;
    w->rows = B;
    return SHARD_OK;
}

}  // namespace

// Scratch of shard_decode_static: part of the library's device image, so no call ever allocates
// it.  In host code this name is only a handle for hipGetSymbolAddress - the address kernels get
// is the one that call returns, looked up once per device in shard_create.
static __device__ __align__(256) unsigned char scratch[SHARD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SHARD_E_HIP, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(SHARD_E_HIP, "hipGetSymbolAddress returned a null address for the static scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SHARD_OK;
}

// Body shared by shard_prefill, shard_decode and shard_decode_static: validate, reserve pages,
// enqueue, and only then commit the new lengths; any failure restores the page bookkeeping.
int run_call(shard* s, const int32_t* seq_ids, int B, int T, bool decode, bool static_ws, const void* x_in, void* x_out,
             void* hip_stream) {
    SeqBatch sb;
    int rc = check_batch(s, seq_ids, B, T, decode, &sb);
    if (rc) return rc;
    if (!x_in || !x_out) return fail(SHARD_E_INVAL, "null activation pointer");
    rc = range_check(s);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    shard::Work local{};
    shard::Work* wk = nullptr;
    if (static_ws) {
        if (s->timing.on) return fail(SHARD_E_STATE, "shard_decode_static cannot run while kernel timing is enabled (it creates events)");
        if (s->record_layers) return fail(SHARD_E_STATE, "shard_decode_static cannot run inside shard_profile");
        rc = carve_static(s, sb, &local);
        if (rc) return rc;
        wk = &local;
    } else {
        rc = acquire_work(s, st, static_cast<size_t>(B) * T, &wk);
        if (rc) return rc;
    }
    (void)hipGetLastError();   // a stale error of the caller's own must not be blamed on this call
    GrowUndo undo(s, sb);
    grow_sequences(s, sb, T, st);
    if (decode) run_decode(s, *wk, sb, static_cast<const float*>(x_in), static_cast<float*>(x_out), st);
    else run_prefill(s, *wk, sb, T, static_cast<const float*>(x_in), static_cast<float*>(x_out), st);
    rc = static_ws ? SHARD_OK : release_work(wk, st);
    if (rc == SHARD_OK) rc = check_launch();
    if (rc) {
        undo.rollback();
        return rc;
    }
    for (int b = 0; b < B; ++b) s->seq_len[sb.seq[b]] += T;
    return SHARD_OK;
}

// Nothing may throw across the C boundary: allocation failures of the host containers map to
// SHARD_E_NOMEM, anything else to SHARD_E_HIP.
template <typename F>
int guarded(F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(SHARD_E_NOMEM, "host allocation failed");
    } catch (const std::exception& e) {
        return fail(SHARD_E_HIP, "unexpected failure: %s", e.what());
    } catch (...) {
        return fail(SHARD_E_HIP, "unexpected failure");
    }
}

}  // namespace

extern "C" {

const char* shard_last_error(void) { return g_err.c_str(); }

static int create_impl(shard_t** out, const shard_model_cfg* model, const shard_kv_cfg* kv, int32_t layer_lo,
                       int32_t layer_hi, const shard_layer_weights* w, int32_t weights_on_device) {
    if (!out) return fail(SHARD_E_INVAL, "null out");
    *out = nullptr;
    int rc = validate_cfg(model, kv, layer_lo, layer_hi);
    if (rc) return rc;
    if (!w) return fail(SHARD_E_INVAL, "null weights");
    const int L = layer_hi - layer_lo;
    for (int i = 0; i < L; ++i) {
        const void* ptrs[] = {w[i].wq, w[i].wk, w[i].wv, w[i].wo, w[i].w_gate, w[i].w_up, w[i].w_down, w[i].g_attn, w[i].g_ffn};
        for (const void* p : ptrs)
            if (!p) return fail(SHARD_E_INVAL, "layer %d has a null tensor", layer_lo + i);
    }
    shard* s = new (std::nothrow) shard();
    if (!s) return fail(SHARD_E_NOMEM, "host allocation failed");
    struct Guard {   // every early return and every exception releases what was built so far
        shard* s;
        ~Guard() { if (s) free_all(s); }
    } guard{s};
    s->m = *model;
    s->kv = *kv;
    s->layer_lo = layer_lo; s->layer_hi = layer_hi; s->L = L;
    s->es = model->weight_dtype == SHARD_F32 ? 4 : 2;
    const int d = model->d_model, dh = model->head_dim, F = model->ffn_dim;
    s->nq = model->n_heads * dh;
    const int nkv = model->n_kv_heads * dh;
    s->nqkv = s->nq + 2 * nkv;
    s->max_pages = (kv->max_seq_len + kv->page_size - 1) / kv->page_size;
    s->n_pages = s->max_pages * kv->max_seqs;
    s->mmax = kv->max_batch_tokens > 0 ? kv->max_batch_tokens : kv->max_seq_len;
    if (s->mmax < SHARD_MAX_BATCH) s->mmax = SHARD_MAX_BATCH;  // decode batches
    s->layers.resize(L);

    const size_t es = s->es;
    const hipMemcpyKind kind = weights_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
#define CREATE_TRY(expr)                                                                      \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(e_ == hipErrorOutOfMemory ? SHARD_E_NOMEM : SHARD_E_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                               \
    } while (0)

    // the word the kernels raise when a value stored as half leaves half's range: pinned host
    // memory mapped into the device, so the runtime reads it without a copy or a wait
    CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&s->oflow), sizeof(uint32_t), hipHostMallocMapped));
    *s->oflow = 0u;
    {
        const int rc_s = static_scratch_of_current_device(&s->static_scratch);
        if (rc_s) return rc_s;
    }

    const size_t page_elems = static_cast<size_t>(model->n_kv_heads) * kv->page_size * dh;
    uint32_t*& cvt_flag = s->cvt_flag;  // owned by the shard, so every failure path releases it
    for (int i = 0; i < L; ++i) {
        LayerDev& l = s->layers[i];
        CREATE_TRY(hipMalloc(&l.wqkv, static_cast<size_t>(s->nqkv) * d * es));
        CREATE_TRY(hipMalloc(&l.wo, static_cast<size_t>(d) * s->nq * es));
        CREATE_TRY(hipMalloc(&l.wgu, static_cast<size_t>(2) * F * d * es));
        CREATE_TRY(hipMalloc(&l.wd, static_cast<size_t>(d) * F * es));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&l.g_attn), d * sizeof(float)));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&l.g_ffn), d * sizeof(float)));
        CREATE_TRY(hipMalloc(&l.k, page_elems * s->n_pages * es));
        CREATE_TRY(hipMalloc(&l.v, page_elems * s->n_pages * es));
        char* qkv = static_cast<char*>(l.wqkv);
        CREATE_TRY(hipMemcpy(qkv, w[i].wq, static_cast<size_t>(s->nq) * d * es, kind));
        CREATE_TRY(hipMemcpy(qkv + static_cast<size_t>(s->nq) * d * es, w[i].wk, static_cast<size_t>(nkv) * d * es, kind));
        CREATE_TRY(hipMemcpy(qkv + static_cast<size_t>(s->nq + nkv) * d * es, w[i].wv, static_cast<size_t>(nkv) * d * es, kind));
        CREATE_TRY(hipMemcpy(l.wo, w[i].wo, static_cast<size_t>(d) * s->nq * es, kind));
        // gate and up rows interleaved: a 2-D copy with twice the destination pitch
        const size_t rowb = static_cast<size_t>(d) * es;
        CREATE_TRY(hipMemcpy2D(l.wgu, 2 * rowb, w[i].w_gate, rowb, rowb, F, kind));
        CREATE_TRY(hipMemcpy2D(static_cast<char*>(l.wgu) + rowb, 2 * rowb, w[i].w_up, rowb, rowb, F, kind));
        CREATE_TRY(hipMemcpy(l.wd, w[i].w_down, static_cast<size_t>(d) * F * es, kind));
        if (model->weight_dtype == SHARD_BF16) {
            // bf16 exists only at the boundary: the matrices live on the device as IEEE half
            if (!cvt_flag) {
                CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&cvt_flag), sizeof(uint32_t)));
                CREATE_TRY(hipMemset(cvt_flag, 0, sizeof(uint32_t)));
            }
            launch_bf16_to_f16(l.wqkv, static_cast<size_t>(s->nqkv) * d, cvt_flag, nullptr);
            launch_bf16_to_f16(l.wo, static_cast<size_t>(d) * s->nq, cvt_flag, nullptr);
            launch_bf16_to_f16(l.wgu, static_cast<size_t>(2) * F * d, cvt_flag, nullptr);
            launch_bf16_to_f16(l.wd, static_cast<size_t>(d) * F, cvt_flag, nullptr);
        }
        CREATE_TRY(hipMemcpy(l.g_attn, w[i].g_attn, d * sizeof(float), kind));
        CREATE_TRY(hipMemcpy(l.g_ffn, w[i].g_ffn, d * sizeof(float), kind));
        if (model->weight_dtype == SHARD_BF16) {
            // W (g * x_hat) = (W diag g) x_hat: the RMSNorm gains become part of the half matrices
            // that consume the normalised vector, and the gains the kernels still multiply by are 1
            launch_scale_columns_f16(l.wqkv, l.g_attn, s->nqkv, d, cvt_flag, nullptr);
            launch_scale_columns_f16(l.wgu, l.g_ffn, 2 * F, d, cvt_flag, nullptr);
            CREATE_TRY(hipDeviceSynchronize());
            const std::vector<float> ones(d, 1.0f);
            CREATE_TRY(hipMemcpy(l.g_attn, ones.data(), d * sizeof(float), hipMemcpyHostToDevice));
            CREATE_TRY(hipMemcpy(l.g_ffn, ones.data(), d * sizeof(float), hipMemcpyHostToDevice));
        }
        // a cache that was never written must still hold finite numbers (masked lanes read it)
        CREATE_TRY(hipMemset(l.k, 0, page_elems * s->n_pages * es));
        CREATE_TRY(hipMemset(l.v, 0, page_elems * s->n_pages * es));
    }

    // cos/sin of pos * theta^(-2i/dh), evaluated in double on the host and rounded once
    {
        std::vector<float2> tab(static_cast<size_t>(kv->max_seq_len) * (dh / 2));
        for (int p = 0; p < kv->max_seq_len; ++p)
            for (int i = 0; i < dh / 2; ++i) {
                const double ang = p * std::pow(static_cast<double>(model->rope_theta), -2.0 * i / dh);
                tab[static_cast<size_t>(p) * (dh / 2) + i] = make_float2(static_cast<float>(std::cos(ang)),
                                                                         static_cast<float>(std::sin(ang)));
            }
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&s->rope), tab.size() * sizeof(float2)));
        CREATE_TRY(hipMemcpy(s->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    }

    const size_t bt_elems = static_cast<size_t>(kv->max_seqs) * s->max_pages;
    CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&s->block_table), bt_elems * sizeof(int32_t)));
    CREATE_TRY(hipMemset(s->block_table, 0, bt_elems * sizeof(int32_t)));
    s->host_table.assign(bt_elems, 0);
    s->free_pages.resize(s->n_pages);
    for (int i = 0; i < s->n_pages; ++i) s->free_pages[i] = i;  // popped from the back: highest page first
    s->seq_len.assign(kv->max_seqs, -1);
    s->seq_pages.assign(kv->max_seqs, 0);

    const size_t units = static_cast<size_t>(SHARD_MAX_BATCH) * model->n_heads;
    for (int wi = 0; wi < SHARD_MAX_STREAMS; ++wi) {
        shard::Work& w = s->work[wi];
        // every set takes a whole prefill when that is cheap (256 MB); otherwise only set 0 does
        const size_t row_bytes = static_cast<size_t>(d) * es + 2ull * s->nq * sizeof(float) + static_cast<size_t>(F) * sizeof(float);
        const bool big = wi == 0 || static_cast<size_t>(s->mmax) * row_bytes <= (256ull << 20);
        const size_t rows = big ? static_cast<size_t>(s->mmax) : static_cast<size_t>(SHARD_MAX_BATCH);
        w.rows = rows;
        CREATE_TRY(hipMalloc(&w.h, rows * d * es));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&w.q), rows * s->nq * sizeof(float)));
        CREATE_TRY(hipMalloc(&w.o, rows * s->nq * sizeof(float)));
        CREATE_TRY(hipMalloc(&w.f, rows * F * sizeof(float)));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&w.part_o), units * s->nsplit_max * dh * sizeof(float)));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&w.part_ml), units * s->nsplit_max * 2 * sizeof(float)));
        CREATE_TRY(hipMalloc(reinterpret_cast<void**>(&w.splitk), SPLITK_FLOATS * sizeof(float)));   // split-K partial sums (prefill GEMM)
        CREATE_TRY(hipEventCreateWithFlags(&w.done, hipEventDisableTiming));
    }
    s->layer_ev.resize(L + 1);
    for (auto& e : s->layer_ev) e = nullptr;
    for (auto& e : s->layer_ev) CREATE_TRY(hipEventCreate(&e));
    CREATE_TRY(hipDeviceSynchronize());
    if (cvt_flag) {
        uint32_t over = 0;
        const hipError_t e1 = hipMemcpy(&over, cvt_flag, sizeof over, hipMemcpyDeviceToHost);
        (void)hipFree(cvt_flag);
        cvt_flag = nullptr;
        if (e1 != hipSuccess || over) {
            return e1 != hipSuccess ? fail(SHARD_E_HIP, "reading the conversion flag: %s", hipGetErrorString(e1))
                                    : fail(SHARD_E_INVAL, "a bf16 weight (times its RMSNorm gain, for wq/wk/wv/w_gate/w_up) exceeds the range of IEEE half (65504)");
        }
    }
#undef CREATE_TRY
    const int rc_l = check_launch();   // the conversion kernels of this create
    if (rc_l) return rc_l;
    guard.s = nullptr;
    *out = s;
    return SHARD_OK;
}

int shard_create(shard_t** out, const shard_model_cfg* model, const shard_kv_cfg* kv, int32_t layer_lo,
                 int32_t layer_hi, const shard_layer_weights* w, int32_t weights_on_device) {
    return guarded([&] { return create_impl(out, model, kv, layer_lo, layer_hi, w, weights_on_device); });
}

int shard_destroy(shard_t* s) {
    if (!s) return SHARD_OK;
    const hipError_t e = hipDeviceSynchronize();
    free_all(s);
    if (e != hipSuccess) return fail(SHARD_E_HIP, "hipDeviceSynchronize: %s", hipGetErrorString(e));
    return SHARD_OK;
}

int shard_seq_alloc(shard_t* s, int32_t* seq_id) {
    if (!s || !seq_id) return fail(SHARD_E_INVAL, "null argument");
    for (int i = 0; i < s->kv.max_seqs; ++i)
        if (s->seq_len[i] < 0) {
            s->seq_len[i] = 0;
            s->seq_pages[i] = 0;
            *seq_id = i;
            return SHARD_OK;
        }
    return fail(SHARD_E_KV_FULL, "all %d sequence slots are live", s->kv.max_seqs);
}

int shard_seq_free(shard_t* s, int32_t seq_id) {
    if (!s) return fail(SHARD_E_INVAL, "null shard");
    if (seq_id < 0 || seq_id >= s->kv.max_seqs || s->seq_len[seq_id] < 0)
        return fail(SHARD_E_STATE, "seq_id %d is not live", seq_id);
    for (int i = s->seq_pages[seq_id] - 1; i >= 0; --i)
        s->free_pages.push_back(s->host_table[static_cast<size_t>(seq_id) * s->max_pages + i]);
    s->seq_pages[seq_id] = 0;
    s->seq_len[seq_id] = -1;
    return SHARD_OK;
}

int32_t shard_seq_len(shard_t* s, int32_t seq_id) {
    if (!s) return fail(SHARD_E_INVAL, "null shard");
    if (seq_id < 0 || seq_id >= s->kv.max_seqs || s->seq_len[seq_id] < 0)
        return fail(SHARD_E_STATE, "seq_id %d is not live", seq_id);
    return s->seq_len[seq_id];
}

int shard_prefill(shard_t* s, const int32_t* seq_ids, int32_t B, int32_t T, const void* x_in, void* x_out,
                  void* hip_stream) {
    return guarded([&] { return run_call(s, seq_ids, B, T, false, false, x_in, x_out, hip_stream); });
}

int shard_decode(shard_t* s, const int32_t* seq_ids, int32_t B, const void* x_in, void* x_out, void* hip_stream) {
    return guarded([&] { return run_call(s, seq_ids, B, 1, true, false, x_in, x_out, hip_stream); });
}

int shard_decode_static(shard_t* s, const int32_t* seq_ids, int32_t B, const void* x_in, void* x_out, void* hip_stream) {
    return guarded([&] { return run_call(s, seq_ids, B, 1, true, true, x_in, x_out, hip_stream); });
}

int shard_overflow(shard_t* s, int32_t clear, int32_t* overflowed) {
    if (!s || !overflowed) return fail(SHARD_E_INVAL, "null argument");
    volatile uint32_t* flag = s->oflow;
    *overflowed = flag && *flag ? 1 : 0;
    if (clear && flag) *flag = 0u;
    return SHARD_OK;
}

int shard_timing_enable(shard_t* s, int32_t on) {
    if (!s) return fail(SHARD_E_INVAL, "null shard");
    Timing& t = s->timing;
    t.on = on != 0;
    for (int k = 0; k < SHARD_K_COUNT; ++k) {
        t.used[k] = 0;
        t.launches[k] = 0;
        t.seconds[k] = 0.0;
    }
    return SHARD_OK;
}

int shard_timing_read(shard_t* s, int64_t launches[SHARD_K_COUNT], double seconds[SHARD_K_COUNT]) {
    if (!s || !launches || !seconds) return fail(SHARD_E_INVAL, "null argument");
    Timing& t = s->timing;
    HIP_TRY(hipDeviceSynchronize());  // timed launches may sit on several streams
    for (int k = 0; k < SHARD_K_COUNT; ++k) {
        for (size_t i = 0; i + 1 < t.used[k]; i += 2) {
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, t.ev[k][i], t.ev[k][i + 1]));
            t.seconds[k] += ms * 1e-3;
            t.launches[k] += 1;
        }
        t.used[k] = 0;
        launches[k] = t.launches[k];
        seconds[k] = t.seconds[k];
    }
    return SHARD_OK;
}

static int profile_impl(shard_t* s, int32_t B, int32_t T_prefill, int32_t n_decode, int32_t iters, shard_layer_profile* out) {
    if (!s || !out) return fail(SHARD_E_INVAL, "null argument");
    if (B < 1 || B > SHARD_MAX_BATCH || T_prefill < 1 || n_decode < 0 || iters < 1)
        return fail(SHARD_E_INVAL, "bad profile shape");
    if (static_cast<long>(B) * T_prefill > s->mmax) return fail(SHARD_E_INVAL, "B*T_prefill exceeds max_batch_tokens");
    if (T_prefill + n_decode > s->kv.max_seq_len) return fail(SHARD_E_KV_FULL, "T_prefill + n_decode > max_seq_len");
    int free_slots = 0;
    for (int v : s->seq_len) free_slots += v < 0;
    if (free_slots < B) return fail(SHARD_E_KV_FULL, "profiling needs %d free sequence slots, %d available", B, free_slots);

    const int d = s->m.d_model, L = s->L;
    const size_t n = static_cast<size_t>(B) * T_prefill * d;
    std::vector<float> hx(n);
    uint32_t lcg = 12345u;  // deterministic activations of unit scale
    for (auto& v : hx) {
        lcg = lcg * 1664525u + 1013904223u;
        v = (static_cast<float>(lcg >> 8) / 8388608.0f - 1.0f) * 1.7320508f;
    }
    float *x = nullptr, *y = nullptr;
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&x), n * sizeof(float)));
    if (hipMalloc(reinterpret_cast<void**>(&y), n * sizeof(float)) != hipSuccess) {
        (void)hipFree(x);
        return fail(SHARD_E_NOMEM, "profile buffers");
    }
    int rc = SHARD_OK;
    std::vector<double> tp(L, 0.0), td(L, 0.0);
    std::vector<int32_t> ids(B);
    auto add_layer_times = [&](std::vector<double>& acc) -> bool {
        if (hipEventSynchronize(s->layer_ev[L]) != hipSuccess) return false;
        for (int i = 0; i < L; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, s->layer_ev[i], s->layer_ev[i + 1]) != hipSuccess) return false;
            acc[i] += ms * 1e-3;
        }
        return true;
    };
    if (hipMemcpy(x, hx.data(), n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) rc = fail(SHARD_E_HIP, "profile upload");
    for (int it = -1; it < iters && rc == SHARD_OK; ++it) {  // iteration -1 is an untimed warm-up
        for (int b = 0; b < B && rc == SHARD_OK; ++b) rc = shard_seq_alloc(s, &ids[b]);
        if (rc) break;
        s->record_layers = true;
        rc = shard_prefill(s, ids.data(), B, T_prefill, x, y, nullptr);
        if (rc == SHARD_OK && it >= 0 && !add_layer_times(tp)) rc = fail(SHARD_E_HIP, "profile events");
        for (int k = 0; k < n_decode && rc == SHARD_OK; ++k) {
            rc = shard_decode(s, ids.data(), B, x, y, nullptr);
            if (rc == SHARD_OK && it >= 0 && !add_layer_times(td)) rc = fail(SHARD_E_HIP, "profile events");
        }
        s->record_layers = false;
        (void)hipDeviceSynchronize();
        for (int b = 0; b < B; ++b) (void)shard_seq_free(s, ids[b]);
    }
    s->record_layers = false;
    (void)hipDeviceSynchronize();
    (void)hipFree(x);
    (void)hipFree(y);
    if (rc) return rc;
    const shard_model_cfg& m = s->m;
    const uint64_t wbytes = (static_cast<uint64_t>(s->nqkv) * d + static_cast<uint64_t>(d) * s->nq +
                             3ull * m.ffn_dim * d) * s->es + 2ull * d * sizeof(float);
    for (int i = 0; i < L; ++i) {
        shard_layer_profile& p = out[i];
        p.t_prefill_s = tp[i] / iters;
        p.t_decode_s = n_decode ? td[i] / (static_cast<double>(iters) * n_decode) : 0.0;
        p.t_avg_s = (p.t_prefill_s + n_decode * p.t_decode_s) / (1 + n_decode);
        p.act_bytes_prefill = static_cast<uint64_t>(B) * T_prefill * d * sizeof(float);
        p.act_bytes_decode = static_cast<uint64_t>(B) * d * sizeof(float);
        p.weight_bytes = wbytes;
        p.kv_bytes_per_token = 2ull * m.n_kv_heads * m.head_dim * s->es;
    }
    return SHARD_OK;
}

int shard_profile(shard_t* s, int32_t B, int32_t T_prefill, int32_t n_decode, int32_t iters, shard_layer_profile* out) {
    return guarded([&] { return profile_impl(s, B, T_prefill, n_decode, iters, out); });
}

// ---- the ends of a model: embedding lookup, final norm + LM head, greedy choice ----------
}  // extern "C"

struct shard_ends {
    shard_model_cfg m{};
    int vocab = 0, max_tokens = 0, dt = DT_F32;
    size_t es = 4;
    void* tok = nullptr;       // [V, d]
    void* lm = nullptr;        // [V, d]
    float* g_final = nullptr;  // [d]
    int32_t* ids_dev = nullptr;
    uint32_t* flag = nullptr;  // conversion overflow / clamped-id flag
};

namespace {
void free_ends(shard_ends* e) {
    void* ptrs[] = {e->tok, e->lm, e->g_final, e->ids_dev, e->flag};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    delete e;
}
}  // namespace

extern "C" {

int shard_ends_create(shard_ends_t** out, const shard_model_cfg* model, int32_t vocab, int32_t max_tokens,
                      const void* tok_embeddings, const float* g_final, const void* lm_head, int32_t weights_on_device) {
    if (!out) return fail(SHARD_E_INVAL, "null out");
    *out = nullptr;
    if (!model) return fail(SHARD_E_INVAL, "null model");
    if (model->d_model < 8 || model->d_model % 8) return fail(SHARD_E_INVAL, "d_model must be a positive multiple of 8");
    if (model->weight_dtype != SHARD_F32 && model->weight_dtype != SHARD_BF16)
        return fail(SHARD_E_INVAL, "unknown weight_dtype %d", model->weight_dtype);
    if (!(model->rms_eps >= 0.f)) return fail(SHARD_E_INVAL, "bad rms_eps");
    if (vocab < 1 || max_tokens < 1) return fail(SHARD_E_INVAL, "vocab and max_tokens must be positive");
    if (!tok_embeddings && !lm_head) return fail(SHARD_E_INVAL, "neither end given");
    if ((g_final == nullptr) != (lm_head == nullptr)) return fail(SHARD_E_INVAL, "g_final and lm_head go together");
    shard_ends* e = new (std::nothrow) shard_ends();
    if (!e) return fail(SHARD_E_NOMEM, "host allocation failed");
    e->m = *model;
    e->vocab = vocab;
    e->max_tokens = max_tokens;
    e->es = model->weight_dtype == SHARD_F32 ? 4 : 2;
    e->dt = model->weight_dtype == SHARD_F32 ? DT_F32 : DT_F16;
    const size_t elems = static_cast<size_t>(vocab) * model->d_model;
    const hipMemcpyKind kind = weights_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
#define ENDS_TRY(expr)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            free_ends(e);                                                                     \
            return fail(e_ == hipErrorOutOfMemory ? SHARD_E_NOMEM : SHARD_E_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                               \
        }                                                                                     \
    } while (0)
    ENDS_TRY(hipMalloc(reinterpret_cast<void**>(&e->flag), sizeof(uint32_t)));
    ENDS_TRY(hipMemset(e->flag, 0, sizeof(uint32_t)));
    if (tok_embeddings) {
        ENDS_TRY(hipMalloc(&e->tok, elems * e->es));
        ENDS_TRY(hipMemcpy(e->tok, tok_embeddings, elems * e->es, kind));
        ENDS_TRY(hipMalloc(reinterpret_cast<void**>(&e->ids_dev), static_cast<size_t>(max_tokens) * sizeof(int32_t)));
        if (model->weight_dtype == SHARD_BF16) launch_bf16_to_f16(e->tok, elems, e->flag, nullptr);
    }
    if (lm_head) {
        ENDS_TRY(hipMalloc(&e->lm, elems * e->es));
        ENDS_TRY(hipMemcpy(e->lm, lm_head, elems * e->es, kind));
        ENDS_TRY(hipMalloc(reinterpret_cast<void**>(&e->g_final), model->d_model * sizeof(float)));
        ENDS_TRY(hipMemcpy(e->g_final, g_final, model->d_model * sizeof(float), kind));
        if (model->weight_dtype == SHARD_BF16) launch_bf16_to_f16(e->lm, elems, e->flag, nullptr);
    }
    ENDS_TRY(hipDeviceSynchronize());
    uint32_t over = 0;
    ENDS_TRY(hipMemcpy(&over, e->flag, sizeof over, hipMemcpyDeviceToHost));
#undef ENDS_TRY
    if (over) {
        free_ends(e);
        return fail(SHARD_E_INVAL, "a bf16 entry of tok_embeddings or lm_head exceeds the range of IEEE half (65504)");
    }
    *out = e;
    return SHARD_OK;
}

int shard_ends_destroy(shard_ends_t* e) {
    if (!e) return SHARD_OK;
    const hipError_t rc = hipDeviceSynchronize();
    free_ends(e);
    if (rc != hipSuccess) return fail(SHARD_E_HIP, "hipDeviceSynchronize: %s", hipGetErrorString(rc));
    return SHARD_OK;
}

int shard_ends_embed(shard_ends_t* e, const int32_t* token_ids, int32_t n, void* x_out, void* hip_stream) {
    if (!e || !token_ids || !x_out) return fail(SHARD_E_INVAL, "null argument");
    if (!e->tok) return fail(SHARD_E_STATE, "this ends object holds no embedding table");
    if (n < 1 || n > e->max_tokens) return fail(SHARD_E_INVAL, "n = %d outside 1..max_tokens (%d)", n, e->max_tokens);
    for (int i = 0; i < n; ++i)
        if (token_ids[i] < 0 || token_ids[i] >= e->vocab)
            return fail(SHARD_E_INVAL, "token_ids[%d] = %d outside the vocabulary (%d)", i, token_ids[i], e->vocab);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (n <= 128) {
        TokenIds ids{};
        ids.n = n;
        for (int i = 0; i < n; ++i) ids.id[i] = token_ids[i];
        launch_embed(e->tok, e->dt, e->vocab, e->m.d_model, &ids, nullptr, n, static_cast<float*>(x_out), e->flag, st);
    } else {
        // the copy from pageable host memory completes (from the host's view) before this returns
        HIP_TRY(hipMemcpyAsync(e->ids_dev, token_ids, static_cast<size_t>(n) * sizeof(int32_t), hipMemcpyHostToDevice, st));
        launch_embed(e->tok, e->dt, e->vocab, e->m.d_model, nullptr, e->ids_dev, n, static_cast<float*>(x_out), e->flag, st);
    }
    return check_launch();
}

int shard_ends_logits(shard_ends_t* e, const void* x, int32_t n, void* logits, void* hip_stream) {
    if (!e || !x || !logits) return fail(SHARD_E_INVAL, "null argument");
    if (!e->lm) return fail(SHARD_E_STATE, "this ends object holds no output projection");
    if (n < 1 || n > SHARD_MAX_BATCH) return fail(SHARD_E_INVAL, "n = %d outside 1..%d", n, SHARD_MAX_BATCH);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    SeqBatch sb{};
    for (int r0 = 0; r0 < n; r0 += 8) {  // the streaming projection takes up to 8 rows per pass
        DecodeLinear d{};
        d.W = e->lm; d.N = e->vocab; d.K = e->m.d_model; d.wt = e->dt;
        d.nb = n - r0 < 8 ? n - r0 : 8;
        d.x = static_cast<const float*>(x) + static_cast<size_t>(r0) * e->m.d_model;
        d.gain = e->g_final; d.eps = e->m.rms_eps; d.epi = EPI_STORE;
        d.out = static_cast<float*>(logits) + static_cast<size_t>(r0) * e->vocab;
        sb.n = d.nb;
        launch_decode_linear(d, sb, st);
    }
    return check_launch();
}

int shard_ends_argmax(shard_ends_t* e, const void* logits, int32_t n, int32_t* token_ids_out, void* hip_stream) {
    if (!e || !logits || !token_ids_out) return fail(SHARD_E_INVAL, "null argument");
    if (n < 1) return fail(SHARD_E_INVAL, "n must be positive");
    launch_argmax(static_cast<const float*>(logits), n, e->vocab, token_ids_out, static_cast<hipStream_t>(hip_stream));
    return check_launch();
}

}  // extern "C"

// ---- introspection of launch decisions (include/shard_introspect.h) -----------------------
extern "C" {

const char* shard_variant_name(int32_t family, int32_t index) {
    switch (family) {
        case SHARD_FAMILY_PREFILL_GEMM: return shk::prefill_gemm_variant_name(index);
        case SHARD_FAMILY_DECODE_STREAM: return shk::decode_linear_variant_name(index);
        case SHARD_FAMILY_DECODE_MFMA: return shk::decode_linear_mfma_variant_name(index);
        default: return nullptr;
    }
}

int32_t shard_variant_prefill_gemm(int32_t weight_dtype, int32_t M, int32_t N, int32_t K, int32_t residual_epilogue,
                                   int32_t* k_slices) {
    if ((weight_dtype != SHARD_F32 && weight_dtype != SHARD_BF16) || M < 1 || N < 1 || K < 1) return -1;
    int ks = 1;
    // O and down projections carry the shard's split-K scratch; QKV and gate/up never split
    const int id = shk::choose_prefill_gemm(weight_dtype == SHARD_F32 ? DT_F32 : DT_F16, M, N, K,
                                            residual_epilogue ? EPI_RESID : EPI_SWIGLU, residual_epilogue != 0, SPLITK_FLOATS, &ks);
    if (k_slices) *k_slices = ks;
    return id;
}

int32_t shard_variant_decode_linear(const shard_model_cfg* model, int32_t B, int32_t N, int32_t K, int32_t* family,
                                    int32_t* rows_per_pass, int32_t* rows_per_workgroup) {
    if (!model || !family || !rows_per_pass || !rows_per_workgroup || B < 1 || B > SHARD_MAX_BATCH || N < 1 || K < 1) return -1;
    if (model->weight_dtype != SHARD_F32 && model->weight_dtype != SHARD_BF16) return -1;
    if (decode_on_matrix_cores(*model, B)) {
        int rows = 0;
        const int id = shk::choose_decode_linear_mfma(N, K, &rows);
        *family = SHARD_FAMILY_DECODE_MFMA;
        *rows_per_pass = B < 16 ? B : 16;
        *rows_per_workgroup = rows;
        return id;
    }
    *family = SHARD_FAMILY_DECODE_STREAM;
    *rows_per_pass = B < 8 ? B : 8;
    *rows_per_workgroup = 0;
    return shk::choose_decode_linear(model->weight_dtype == SHARD_F32 ? DT_F32 : DT_F16, *rows_per_pass, N, K);
}

void shard_test_inject_launch_error(int32_t on) { shk::inject_kernel_attribute_error(on != 0); }

}  // extern "C"
