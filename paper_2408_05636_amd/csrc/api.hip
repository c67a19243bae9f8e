// C ABI of the SpecDiff round (see include/specdiff.h): weight layout, workspace carving, the two
// forward passes and the draft / verify drivers.  Host code only enqueues kernels; every step of
// Algorithm 1 runs on the device.
#include <string.h>

#include <algorithm>
#include <mutex>
#include <string>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "common.h"
#include "philox.hip.h"

using namespace sd;

namespace sd {
launch_hook_t g_launch_hook = nullptr;
void* g_launch_hook_ctx = nullptr;
}  // namespace sd

namespace {

constexpr int kMaxSteps = 256;   // upper limit of T

// ------------------------------------------------------------------------------------------
// weight layout
// ------------------------------------------------------------------------------------------
struct TensorDesc {
    std::string name;
    int64_t rows, cols;
    int elem;
    int64_t off;
};

bool config_ok(const sd_model_config* c) {
    if (!c) return false;
    if (c->arch != SD_ARCH_GPT2 && c->arch != SD_ARCH_LLAMA) return false;
    if (c->dtype != SD_DTYPE_F32 && c->dtype != SD_DTYPE_BF16) return false;
    if (c->n_layer <= 0 || c->d_model <= 0 || c->n_head <= 0 || c->n_kv_head <= 0 || c->d_ff <= 0 || c->vocab <= 0 ||
        c->n_ctx <= 0)
        return false;
    if (c->d_model % c->n_head || c->n_head % c->n_kv_head) return false;
    const int dh = c->d_model / c->n_head;
    if (dh != 32 && dh != 64 && dh != 128) return false;
    if (c->d_model % 16 || c->d_ff % 16) return false;
    if (c->d_model > 8192) return false;
    if (c->bidirectional && c->arch != SD_ARCH_GPT2) return false;
    if (c->vocab > kChunk * 512) return false;
    return true;
}

void build_layout(const sd_model_config& c, std::vector<TensorDesc>& out, int64_t& total) {
    const int ew = c.dtype == SD_DTYPE_BF16 ? 2 : 4;
    const int64_t d = c.d_model, F = c.d_ff, dkv = (int64_t)c.n_kv_head * (c.d_model / c.n_head);
    int64_t off = 0;
    auto add = [&](const std::string& name, int64_t rows, int64_t cols, int elem) {
        out.push_back(TensorDesc{name, rows, cols, elem, off});
        off = align_up(off + rows * cols * elem, 256);
    };
    add("wte", c.vocab + (c.bidirectional ? 1 : 0), d, ew);
    if (c.arch == SD_ARCH_GPT2) add("wpe", c.n_ctx, d, ew);
    if (c.bidirectional) {
        add("t_w1", d, d, ew); add("t_b1", 1, d, 4);
        add("t_w2", d, d, ew); add("t_b2", 1, d, 4);
    }
    for (int i = 0; i < c.n_layer; ++i) {
        const std::string p = "l" + std::to_string(i) + ".";
        if (c.arch == SD_ARCH_GPT2) {
            add(p + "ln1_g", 1, d, 4); add(p + "ln1_b", 1, d, 4);
            add(p + "w_qkv", d + 2 * dkv, d, ew); add(p + "b_qkv", 1, d + 2 * dkv, 4);
            add(p + "w_o", d, d, ew); add(p + "b_o", 1, d, 4);
            add(p + "ln2_g", 1, d, 4); add(p + "ln2_b", 1, d, 4);
            add(p + "w_fc", F, d, ew); add(p + "b_fc", 1, F, 4);
            add(p + "w_proj", d, F, ew); add(p + "b_proj", 1, d, 4);
        } else {
            add(p + "ln1_g", 1, d, 4);
            add(p + "w_qkv", d + 2 * dkv, d, ew);
            add(p + "w_o", d, d, ew);
            add(p + "ln2_g", 1, d, 4);
            add(p + "w_gate", F, d, ew);
            add(p + "w_up", F, d, ew);
            add(p + "w_proj", d, F, ew);
        }
    }
    add("lnf_g", 1, d, 4);
    if (c.arch == SD_ARCH_GPT2) add("lnf_b", 1, d, 4);
    add("w_head", c.vocab, d, ew);
    total = off;
}

struct Layer {
    const float *ln1_g = nullptr, *ln1_b = nullptr, *b_qkv = nullptr, *b_o = nullptr, *ln2_g = nullptr, *ln2_b = nullptr,
                *b_fc = nullptr, *b_proj = nullptr;
    const void *w_qkv = nullptr, *w_o = nullptr, *w_fc = nullptr, *w_proj = nullptr;   // w_fc: [F,d] or gate|up [2F,d]
    // LayerNorm folded into the next contraction: u = W g, v = W beta + bias (device, computed at creation)
    float *fu_qkv = nullptr, *fv_qkv = nullptr, *fu_fc = nullptr, *fv_fc = nullptr;
};

struct Model {
    sd_model_config c;
    int dh, dq, dkv, ld, ew;
    const void *wte = nullptr, *wpe = nullptr, *t_w1 = nullptr, *t_w2 = nullptr, *w_head = nullptr;
    const float *t_b1 = nullptr, *t_b2 = nullptr, *lnf_g = nullptr, *lnf_b = nullptr;
    float *fu_head = nullptr, *fv_head = nullptr;   // final LayerNorm folded into the LM head: u = W g, v = W beta
    std::vector<Layer> L;
    bool fold = false;       // norms in front of QKV / MLP-up are folded into those contractions
    void *kcache = nullptr, *vcache = nullptr;   // causal models: [layer][sequence][n_ctx][n_kv_head * d_head] each
};

bool bind_model(Model& m, const sd_model_config& c, const void* base) {
    m.c = c;
    m.dh = c.d_model / c.n_head;
    m.dq = c.d_model;
    m.dkv = c.n_kv_head * m.dh;
    m.ld = vocab_pad(c.vocab);
    m.ew = c.dtype == SD_DTYPE_BF16 ? 2 : 4;
    m.L.assign(c.n_layer, Layer());
    std::vector<TensorDesc> t;
    int64_t total;
    build_layout(c, t, total);
    const char* b = static_cast<const char*>(base);
    for (const TensorDesc& d : t) {
        const void* p = b + d.off;
        const float* f = reinterpret_cast<const float*>(p);
        const std::string& n = d.name;
        if (n == "wte") m.wte = p;
        else if (n == "wpe") m.wpe = p;
        else if (n == "t_w1") m.t_w1 = p;
        else if (n == "t_b1") m.t_b1 = f;
        else if (n == "t_w2") m.t_w2 = p;
        else if (n == "t_b2") m.t_b2 = f;
        else if (n == "lnf_g") m.lnf_g = f;
        else if (n == "lnf_b") m.lnf_b = f;
        else if (n == "w_head") m.w_head = p;
        else {
            const size_t dot = n.find('.');
            if (n[0] != 'l' || dot == std::string::npos) return false;
            Layer& l = m.L[std::stoi(n.substr(1, dot - 1))];
            const std::string s = n.substr(dot + 1);
            if (s == "ln1_g") l.ln1_g = f;
            else if (s == "ln1_b") l.ln1_b = f;
            else if (s == "w_qkv") l.w_qkv = p;
            else if (s == "b_qkv") l.b_qkv = f;
            else if (s == "w_o") l.w_o = p;
            else if (s == "b_o") l.b_o = f;
            else if (s == "ln2_g") l.ln2_g = f;
            else if (s == "ln2_b") l.ln2_b = f;
            else if (s == "w_fc" || s == "w_gate") l.w_fc = p;     // w_up follows w_gate contiguously
            else if (s == "w_up") {
                if (static_cast<const char*>(p) != static_cast<const char*>(l.w_fc) + (int64_t)c.d_ff * c.d_model * m.ew)
                    return false;
            } else if (s == "b_fc") l.b_fc = f;
            else if (s == "w_proj") l.w_proj = p;
            else if (s == "b_proj") l.b_proj = f;
            else return false;
        }
    }
    return true;
}

// ------------------------------------------------------------------------------------------
// workspace
// ------------------------------------------------------------------------------------------
struct Arena {
    char* base;
    int64_t off = 0;
    explicit Arena(void* b) : base(static_cast<char*>(b)) {}
    template <typename T> T* take(int64_t count, int64_t elem = sizeof(T)) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off = align_up(off + count * elem, 256);
        return p;
    }
};

struct Buffers {
    float* h; void* xn; void* qkv; void* att; void* mlp; void* act; void* xf;
    float *logits_d, *logits_t, *q, *qtok, *temb, *temb_hidden;
    float* rope_cs;          // (cos, sin) of the rotation angles of the target's query rows, [rows][d_head / 2][2]
    int32_t *z, *n_acc, *tok;
    char* maps[3];           // packed row maps: 0 drafter, 1 target query rows, 2 target prefill
    uint64_t* seed;          // Philox key of the current call
    void* sample_scratch;
    float *fold_t, *fold_d;  // folded-norm vectors of the target / drafter layers
    float* stats;            // partial row sums (sum h, sum h^2) of the residual stream, [rows][parts][2]
    SplitWorkspace split;    // tickets + partial sums of the contractions that split K over workgroups
    void *kcache, *vcache;
};

struct Limits { int64_t max_rows, rows_head, dmax, qkvmax, ffmax, ew; int64_t prefix_cap; int64_t map_bytes; };

Limits limits_of(const sd_model_config& t, const sd_model_config& d, int max_batch, int gamma_max) {
    Limits l;
    l.max_rows = (int64_t)max_batch * (t.n_ctx > d.n_ctx ? t.n_ctx : d.n_ctx);
    l.rows_head = (int64_t)max_batch * (gamma_max + 1);
    l.dmax = t.d_model > d.d_model ? t.d_model : d.d_model;
    auto qkvw = [](const sd_model_config& c) { return (int64_t)c.d_model + 2 * (int64_t)c.n_kv_head * (c.d_model / c.n_head); };
    auto ffw = [](const sd_model_config& c) { return (int64_t)c.d_ff * (c.arch == SD_ARCH_LLAMA ? 2 : 1); };
    l.qkvmax = qkvw(t) > qkvw(d) ? qkvw(t) : qkvw(d);
    l.ffmax = ffw(t) > ffw(d) ? ffw(t) : ffw(d);
    l.ew = (t.dtype == SD_DTYPE_F32 || d.dtype == SD_DTYPE_F32) ? 4 : 2;
    l.prefix_cap = l.max_rows;
    const int64_t max_heads = t.n_head > d.n_head ? t.n_head : d.n_head;
    const int64_t order_cap = 8 * (l.max_rows / 32 + max_batch + 1) * max_heads;      // attention launch order, see upload_rows
    l.map_bytes = align_up((l.prefix_cap + 4 * l.max_rows + (int64_t)max_batch * gamma_max) * 4 + 32 + l.max_rows * 8 +
                           l.max_rows * (int64_t)sizeof(AttnTile) + 32 + 2 * order_cap * 4, 256);
    return l;
}

// floats needed for the folded LayerNorm vectors of a model (u and v for QKV and MLP-up of every layer and for the LM head)
constexpr int64_t kSplitBytes = kSplitTicketBytes + (64 << 20);

int64_t fold_floats(const sd_model_config& c) {
    if (c.arch != SD_ARCH_GPT2 || c.dtype != SD_DTYPE_BF16) return 64;
    const int64_t qkv = (int64_t)c.d_model + 2 * (int64_t)c.n_kv_head * (c.d_model / c.n_head);
    return (int64_t)c.n_layer * 2 * (align_up(qkv, 64) + align_up(c.d_ff, 64)) + 2 * align_up(c.vocab, 64);
}

int64_t carve(Arena& a, Buffers& b, const sd_model_config& t, const sd_model_config& d, int max_batch, int gamma_max) {
    const Limits l = limits_of(t, d, max_batch, gamma_max);
    const int64_t ld = vocab_pad(t.vocab);
    b.h = a.take<float>(l.max_rows * l.dmax);
    b.xn = a.take<char>(l.max_rows * l.dmax, l.ew);
    b.qkv = a.take<char>(l.max_rows * l.qkvmax, l.ew);
    b.att = a.take<char>(l.max_rows * l.dmax, l.ew);
    b.mlp = a.take<char>(l.max_rows * l.ffmax, l.ew);
    b.act = a.take<char>(t.arch == SD_ARCH_LLAMA ? l.max_rows * t.d_ff : 1, l.ew);
    b.xf = a.take<char>(l.rows_head * l.dmax, l.ew);
    b.logits_d = a.take<float>((int64_t)max_batch * gamma_max * ld);
    b.logits_t = a.take<float>(l.rows_head * ld);
    b.q = a.take<float>((int64_t)max_batch * gamma_max * ld);
    b.qtok = a.take<float>((int64_t)max_batch * gamma_max);
    b.rope_cs = a.take<float>(l.rows_head * (int64_t)(t.d_model / t.n_head));
    b.temb = a.take<float>((int64_t)kMaxSteps * d.d_model);
    b.temb_hidden = a.take<float>((int64_t)kMaxSteps * d.d_model);
    b.z = a.take<int32_t>((int64_t)max_batch * gamma_max);
    b.n_acc = a.take<int32_t>(max_batch);
    b.tok = a.take<int32_t>(max_batch);
    for (int i = 0; i < 3; ++i) b.maps[i] = a.take<char>(l.map_bytes);
    b.seed = a.take<uint64_t>(32);
    b.sample_scratch = a.take<char>(sampling_scratch_bytes((int)l.rows_head, t.vocab));
    b.fold_t = a.take<float>(fold_floats(t));
    b.stats = a.take<float>(l.max_rows * ((l.dmax + 31) / 32) * 2);
    b.split.bytes = kSplitBytes;
    b.split.base = a.take<char>(kSplitBytes);
    b.fold_d = a.take<float>(fold_floats(d));
    const int64_t cache = (int64_t)t.n_layer * max_batch * t.n_ctx * t.n_kv_head * (t.d_model / t.n_head);
    b.kcache = a.take<char>(cache, t.dtype == SD_DTYPE_BF16 ? 2 : 4);
    b.vcache = a.take<char>(cache, t.dtype == SD_DTYPE_BF16 ? 2 : 4);
    return a.off;
}

}  // namespace

// Row maps of one forward pass, packed into one device buffer (one upload per call):
// prefix tokens, per row: token source, position, sequence, visible key count, key offset;
// per query tile: first row, row count; per block slot: its row.
struct MapSet {
    int32_t *tokens = nullptr, *src = nullptr, *pos = nullptr, *seq = nullptr, *kvl = nullptr, *blk = nullptr;
    int64_t* kv_off = nullptr;
    AttnTile* tiles = nullptr;
    int32_t* order = nullptr;            // attention workgroup -> tile | head << 20 (or -1), see upload_rows
    int n_order = 0;
    int32_t* groups = nullptr;           // attention workgroup -> up to four tiles of one sequence and head (AttnArgs::groups)
    int n_groups = 0, group_tiles = 0;
    int rows = 0, n_tiles = 0, max_kv = 0;
    int head_row0 = -1;                  // first of the rows the LM head reads when they are one contiguous run, else -1
    int regular = 0;                     // one sequence whose rows all see all keys (AttnArgs::regular)
    int causal_base = -1;                // one sequence at cache row 0 whose query row q sees causal_base + q keys, else -1
    int64_t kv_row0 = -1;                // target query rows of a single sequence: the KV-cache row of row 0 (row r goes to kv_row0 + r), else -1
    bool grouped = false;                // the attention launch order groups sequences per XCD (else it is the plain order)
    double kv_sum = 0, kv_rows = 0;     // sum of kv_len over rows; distinct key rows
    int64_t bytes = -1;
};

// ------------------------------------------------------------------------------------------
// per-kernel timing with HIP events on the handle's stream (off unless sd_profile_begin was called)
// ------------------------------------------------------------------------------------------
struct ProfEntry {
    std::string name;
    int64_t launches = 0;
    double ms = 0.0, bytes = 0.0, flops = 0.0;
};
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> events;      // pairs (start, stop)
    size_t used = 0;
    size_t scope_first = 0;              // first event of the SD_LAUNCH scope that is open
    std::vector<int> pending;            // entry index per used pair
    std::vector<ProfEntry> entries;
    const char* phase = "";              // prefix of the entry names: which part of the round is being enqueued
};

// ------------------------------------------------------------------------------------------
// handle
// ------------------------------------------------------------------------------------------
struct sd_handle {
    Profiler prof;
    Model target, drafter;
    Buffers buf;
    Limits lim;
    int max_batch, gamma_max;
    hipStream_t st;
    // pinned host staging
    char* stage_maps[3] = {nullptr, nullptr, nullptr};   // host images of the packed row maps
    uint64_t* stage_seed = nullptr;
    int32_t* stage_z = nullptr;   // block / draft tokens going to the device
    int32_t* stage_out = nullptr; // results read back
    float* stage_f = nullptr;
    MapSet maps[3];               // what each device map buffer currently holds
    std::vector<char> map_shadow[3];
    // captured launch sequences, keyed by everything that shapes them
    std::unordered_map<uint64_t, hipGraphExec_t> graphs;
    std::unordered_set<uint64_t> seen;   // launch sequences run once so far (captured on their second use)
    bool use_graphs = true;
    int64_t graph_replays = 0;           // launch sequences sent as a graph replay since creation
    int64_t graph_eager = 0;             // launch sequences that ran as eager launches although replay was wanted (first sight of a key excluded)
    int graph_failures = 0;              // captures or instantiations that failed (replay is switched off after the first)
    std::string graph_error;             // what failed
    bool greedy = false;                 // temperature 0 instead of the stochastic rule
    bool skip_idle_steps = false;        // leave out the drafter forwards of steps that reveal no slot (sd_set_step_skipping)
    bool last_draft_sps = false;         // the last drafting call was sd_sps_draft
    int steps_run = 0;                   // drafter forwards of the last sd_draft / sd_round
    int temb_T = 0;                      // number of steps the timestep-embedding table in the workspace was built for
    int target_tiles = 0;                // > 0: the last target pass left per-tile arg-maxima (that many tiles per row) instead of logits
    bool head_folded = false;            // the last run_layers left x and row sums for the final normalisation (run_head folds it)
    // KV-cache state per sequence: number of cached positions and a hash of their tokens
    std::vector<int32_t> cached_len;
    std::vector<uint64_t> cached_hash, cached_fnv;
    // what the last verification scored, for sd_commit: per sequence the prefix length and its last token, and the draft
    int pend_batch = 0, pend_gamma = 0;
    std::vector<int32_t> pend_len, pend_tail, pend_draft;
    // Standard speculative decoding (sd_sps_attach): a small causal drafter with a KV cache of its own
    bool has_sps = false;
    Model sps;
    std::vector<int32_t> sps_cached_len;      // per sequence: positions of the drafter's cache that hold tokens of ...
    std::vector<uint64_t> sps_cached_fnv;     // ... a token string with this running hash
    int64_t sps_map_cap = 0;                  // bytes of one step's row maps
    std::vector<char*> sps_dev, sps_stage;    // row maps: slot 0 = catch-up rows, slot 1 + k = step k (device / pinned host)
    std::vector<MapSet> sps_ms;
    std::vector<std::vector<char>> sps_shadow;
    bool pend_sps = false;                    // the pending verification's draft came from the autoregressive drafter
    std::string err;
};

namespace {

#define SD_HIP(h, expr)                                                                           \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) {                                                                   \
            (h)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                         \
            return SD_ERR_HIP;                                                                    \
        }                                                                                         \
    } while (0)

// One SD_LAUNCH scope = one entry of the profile (a launcher may start several kernels: their times add up).
void prof_hook(void* ctx, hipEvent_t* start, hipEvent_t* stop) {
    sd_handle* h = static_cast<sd_handle*>(ctx);
    Profiler& p = h->prof;
    if (p.used + 2 > p.events.size()) {
        for (int i = 0; i < 2; ++i) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) { *start = *stop = nullptr; return; }
            p.events.push_back(e);
        }
    }
    *start = p.events[p.used];
    *stop = p.events[p.used + 1];
    p.used += 2;
}

void prof_start(sd_handle* h) {
    Profiler& p = h->prof;
    if (!p.on) return;
    p.scope_first = p.used;
    sd::g_launch_hook_ctx = h;
    sd::g_launch_hook = prof_hook;
}

void prof_stop(sd_handle* h, const char* name, double bytes, double flops) {
    Profiler& p = h->prof;
    if (!p.on) return;
    sd::g_launch_hook = nullptr;
    const std::string key = std::string(p.phase) + name;
    int idx = -1;
    for (size_t i = 0; i < p.entries.size(); ++i)
        if (p.entries[i].name == key) { idx = (int)i; break; }
    if (idx < 0) { p.entries.push_back(ProfEntry()); idx = (int)p.entries.size() - 1; p.entries[idx].name = key; }
    p.entries[idx].launches += 1;
    p.entries[idx].bytes += bytes;
    p.entries[idx].flops += flops;
    for (size_t e = p.scope_first; e < p.used; e += 2) p.pending.push_back(idx);
}

// After a stream synchronisation: fold the kernel times of the recorded pairs into the entries.
void prof_flush(sd_handle* h) {
    Profiler& p = h->prof;
    for (size_t i = 0; i < p.pending.size(); ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.events[2 * i], p.events[2 * i + 1]) == hipSuccess) p.entries[p.pending[i]].ms += ms;
    }
    p.pending.clear();
    p.used = 0;
}

// Launch with optional per-kernel timing.  NAME may be assigned by the launcher (kernel variant).
#define SD_LAUNCH(h, NAME, BYTES, FLOPS, expr)                                                    \
    do {                                                                                          \
        prof_start(h);                                                                            \
        hipError_t e_ = (expr);                                                                   \
        prof_stop(h, NAME, (double)(BYTES), (double)(FLOPS));                                     \
        if (e_ != hipSuccess) {                                                                   \
            (h)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                         \
            return SD_ERR_HIP;                                                                    \
        }                                                                                         \
    } while (0)

int sync_stream(sd_handle* h) {
    SD_HIP(h, hipStreamSynchronize(h->st));
    if (h->prof.on || !h->prof.pending.empty()) prof_flush(h);
    return SD_OK;
}

int fail(sd_handle* h, int code, const std::string& msg) {
    if (h) h->err = msg;
    return code;
}

constexpr uint64_t kFnvBasis = 1469598103934665603ull;
uint64_t fnv_extend(uint64_t x, const int32_t* t, int n) {
    for (int i = 0; i < n; ++i) { x ^= (uint32_t)t[i]; x *= 1099511628211ull; }
    return x;
}
uint64_t hash_tokens(const int32_t* t, int n) { return fnv_extend(kFnvBasis, t, n) ^ (uint64_t)n; }

// Validate a ragged batch; returns total token count through *total.
int check_batch(sd_handle* h, int batch, const int32_t* tokens, const int32_t* len, int vocab_limit, int64_t* total) {
    if (!h) return SD_ERR_ARG;
    if (!tokens || !len) return fail(h, SD_ERR_ARG, "null token or length array");
    if (batch <= 0 || batch > h->max_batch) return fail(h, SD_ERR_SHAPE, "batch outside [1, max_batch]");
    int64_t n = 0;
    for (int b = 0; b < batch; ++b) {
        if (len[b] <= 0) return fail(h, SD_ERR_SHAPE, "sequence length must be positive");
        n += len[b];
    }
    if (n > h->lim.prefix_cap) return fail(h, SD_ERR_SHAPE, "batch has more tokens than the workspace holds");
    for (int64_t i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= vocab_limit) return fail(h, SD_ERR_TOKEN, "token id outside the vocabulary");
    *total = n;
    return SD_OK;
}

// Build and upload the packed row maps of one forward.  mode 0: drafter over prefix o block;
// 1: target query rows (last prefix token + gamma draft tokens); 2: target prefill rows [0, L-1);
// 3: step k of the autoregressive drafter (one row per sequence: position L - 1 + k, whose token is the last prefix
// token for k = 0 and draft token k - 1 otherwise); 4: rows [start[b], L - 1) of the autoregressive drafter (the part
// of the prefix its cache does not hold yet).
// The upload is skipped when the device buffer already holds exactly these maps (same prefix,
// same shapes as the previous call of this mode).
int upload_rows(sd_handle* h, int mode, int batch, const int32_t* tokens, const int32_t* len, int64_t n_tokens,
                int gamma, int k = 0, const int32_t* start = nullptr) {
    const Model& m = mode == 0 ? h->drafter : (mode >= 3 ? h->sps : h->target);
    auto rows_of = [&](int b) -> int64_t {
        switch (mode) {
            case 0: return len[b] + gamma;
            case 1: return gamma + 1;
            case 2: return len[b] - 1;
            case 3: return 1;
            default: return len[b] - 1 - start[b];
        }
    };
    int64_t rows = 0, n_tiles = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t rb = rows_of(b);
        rows += rb;
        n_tiles += (rb + 31) / 32;
    }
    if (rows > h->lim.max_rows) return fail(h, SD_ERR_SHAPE, "more rows than the workspace holds");
    const int64_t n_blk = mode == 0 ? (int64_t)batch * gamma : 0;
    // packed layout
    int64_t o = 0;
    auto take = [&](int64_t n) { const int64_t at = o; o += n * 4; return at; };
    const int64_t o_tok = take(n_tokens), o_src = take(rows), o_pos = take(rows), o_seq = take(rows), o_kvl = take(rows),
                  o_blk = take(n_blk);
    o = align_up(o, 16);
    const int64_t o_off = o;
    o += rows * 8;
    o = align_up(o, 16);
    const int64_t o_tiles = o;
    o += n_tiles * (int64_t)sizeof(AttnTile);
    o = align_up(o, 16);
    const int64_t o_order = o;            // filled below, its size depends on the grouping
    const int sps_slot = mode == 3 ? 1 + k : 0;
    char* hb = mode >= 3 ? h->sps_stage[sps_slot] : h->stage_maps[mode];
    const int64_t map_cap = mode == 3 ? h->sps_map_cap : h->lim.map_bytes;
    // Attention launch order.  Workgroups go to the 8 XCDs round-robin by linear id and every XCD has its own
    // L2.  Query tiles and query heads that read the same keys and values (one sequence, one KV head) are
    // placed back to back on one XCD, so that K and V are fetched into one L2 once instead of into all of
    // them by turns: the list of (sequence, KV head, query head, tile) in that order is cut into eight
    // consecutive pieces of equal work (key blocks walked, plus a constant per workgroup), one per XCD --
    // a KV head then lands in at most two L2s, and no XCD gets more than its share (dealing out whole KV
    // heads leaves half the chip idle when 12 heads meet 8 XCDs).  When all keys and values fit any L2
    // anyway the plain order is used.
    const int n_kv_groups = m.c.n_kv_head, q_per_kv = m.c.n_head / m.c.n_kv_head;
    std::vector<std::vector<int32_t>> per_xcd(8), grp_xcd(8);
    int group_tiles = 0;
    bool grouped_order = false;
    {
        double kv_bytes = 0;
        auto kv_of = [&](int b) { return (int64_t)(mode == 2 || mode == 4 ? len[b] - 1 : len[b] + gamma); };
        for (int b = 0; b < batch; ++b) kv_bytes += 2.0 * m.ew * m.dkv * kv_of(b);
        const bool grouped = kv_bytes > 2.0e6;
        grouped_order = grouped;
        auto work_of = [&](int b) { return (kv_of(b) + 31) / 32 + 2; };
        int64_t total = 0, total_grp = 0;
        for (int b = 0; b < batch; ++b) {
            const int64_t ntb = (rows_of(b) + 31) / 32;
            total += work_of(b) * ntb * m.c.n_head;
            total_grp += work_of(b) * ((ntb + 3) / 4) * m.c.n_head;
        }
        int64_t t0 = 0, lin = 0, done = 0, done_grp = 0;
        for (int b = 0; b < batch; ++b) {
            const int64_t rb = rows_of(b);
            const int64_t ntb = (rb + 31) / 32;
            const int64_t wk = work_of(b);
            for (int g = 0; g < n_kv_groups; ++g)
                for (int qh = 0; qh < q_per_kv; ++qh)
                    for (int64_t t = 0; t < ntb; ++t, ++lin, done += wk)
                        per_xcd[grouped ? (8 * done + 4 * wk) / total % 8 : lin % 8].push_back((int32_t)(t0 + t) | ((g * q_per_kv + qh) << 20));
            // the same work as groups of up to four consecutive tiles (they share the sequence's keys)
            for (int g = 0; g < n_kv_groups; ++g)
                for (int qh = 0; qh < q_per_kv; ++qh)
                    for (int64_t t = 0; t < ntb; t += 4, done_grp += wk) {
                        const int n = (int)(ntb - t < 4 ? ntb - t : 4);
                        group_tiles = n > group_tiles ? n : group_tiles;
                        grp_xcd[(8 * done_grp + 4 * wk) / total_grp % 8].push_back((int32_t)(t0 + t) | ((n - 1) << 18) | ((g * q_per_kv + qh) << 20));
                    }
            t0 += ntb;
        }
    }
    size_t per_max = 0;
    for (auto& v : per_xcd) per_max = v.size() > per_max ? v.size() : per_max;
    const int64_t n_order = 8 * (int64_t)per_max;
    o += n_order * 4;
    size_t grp_max = 0;
    for (auto& v : grp_xcd) grp_max = v.size() > grp_max ? v.size() : grp_max;
    const int64_t o_groups = o, n_groups = 8 * (int64_t)grp_max;
    o += n_groups * 4;
    const int64_t bytes = o;
    if (bytes > map_cap || n_tiles >= (1 << 18)) return fail(h, SD_ERR_SHAPE, "row maps exceed the workspace");
    int32_t *s_tok = (int32_t*)(hb + o_tok), *s_src = (int32_t*)(hb + o_src), *s_pos = (int32_t*)(hb + o_pos),
            *s_seq = (int32_t*)(hb + o_seq), *s_kvl = (int32_t*)(hb + o_kvl), *s_blk = (int32_t*)(hb + o_blk);
    int64_t* s_off = (int64_t*)(hb + o_off);
    AttnTile* s_tiles = (AttnTile*)(hb + o_tiles);
    memset(hb, 0, bytes);                                 // padding bytes take part in the "unchanged" comparison
    memcpy(s_tok, tokens, n_tokens * sizeof(int32_t));
    {
        int32_t* s_order = (int32_t*)(hb + o_order);
        for (int64_t j = 0; j < (int64_t)per_max; ++j)
            for (int x = 0; x < 8; ++x) s_order[j * 8 + x] = j < (int64_t)per_xcd[x].size() ? per_xcd[x][j] : -1;
        int32_t* s_groups = (int32_t*)(hb + o_groups);
        for (int64_t j = 0; j < (int64_t)grp_max; ++j)
            for (int x = 0; x < 8; ++x) s_groups[j * 8 + x] = j < (int64_t)grp_xcd[x].size() ? grp_xcd[x][j] : -1;
    }
    int64_t r = 0, tok_off = 0, nt = 0;
    int max_kv = 0;
    double kv_sum = 0, kv_rows = 0;
    for (int b = 0; b < batch; ++b) {
        const int L = len[b];
        const int64_t seq_row0 = r;
        if (mode == 0) {
            const int S = L + gamma;
            for (int p = 0; p < S; ++p, ++r) {
                s_src[r] = p < L ? (int32_t)(tok_off + p) : -(b * gamma + (p - L)) - 1;
                s_pos[r] = p;
                s_seq[r] = b;
                s_kvl[r] = S;
                s_off[r] = seq_row0 * (int64_t)(m.dq + 2 * m.dkv);
                if (p >= L) s_blk[b * gamma + (p - L)] = (int32_t)r;
            }
            if (S > max_kv) max_kv = S;
            kv_sum += (double)S * S;
            kv_rows += S;
        } else if (mode == 1) {
            for (int k = 0; k <= gamma; ++k, ++r) {
                s_src[r] = k == 0 ? (int32_t)(tok_off + L - 1) : -(b * gamma + k - 1) - 1;
                s_pos[r] = L - 1 + k;
                s_seq[r] = b;
                s_kvl[r] = L + k;
                s_off[r] = (int64_t)b * m.c.n_ctx * m.dkv;
                kv_sum += L + k;
            }
            if (L + gamma > max_kv) max_kv = L + gamma;
            kv_rows += L + gamma;
        } else if (mode == 3) {
            s_src[r] = k == 0 ? (int32_t)(tok_off + L - 1) : -(b * gamma + k - 1) - 1;
            s_pos[r] = L - 1 + k;
            s_seq[r] = b;
            s_kvl[r] = L + k;
            s_off[r] = (int64_t)b * m.c.n_ctx * m.dkv;
            kv_sum += L + k;
            ++r;
            if (L + k > max_kv) max_kv = L + k;
            kv_rows += L + k;
        } else {
            for (int p = mode == 4 ? start[b] : 0; p < L - 1; ++p, ++r) {
                s_src[r] = (int32_t)(tok_off + p);
                s_pos[r] = p;
                s_seq[r] = b;
                s_kvl[r] = p + 1;
                s_off[r] = (int64_t)b * m.c.n_ctx * m.dkv;
                kv_sum += p + 1;
            }
            if (L - 1 > max_kv) max_kv = L - 1;
            kv_rows += L - 1;
        }
        for (int64_t t0 = seq_row0; t0 < r; t0 += 32) {      // query tiles never span two sequences
            AttnTile& tl = s_tiles[nt++];
            tl.row0 = (int32_t)t0;
            tl.nrows = (int32_t)(r - t0 < 32 ? r - t0 : 32);
            tl.kv_max = 0;
            for (int q = 0; q < tl.nrows; ++q) tl.kv_max = s_kvl[t0 + q] > tl.kv_max ? s_kvl[t0 + q] : tl.kv_max;
            tl.kv_off = s_off[t0];
        }
        tok_off += L;
    }
    MapSet& ms = mode >= 3 ? h->sps_ms[sps_slot] : h->maps[mode];
    std::vector<char>& shadow = mode >= 3 ? h->sps_shadow[sps_slot] : h->map_shadow[mode];
    char* db = mode >= 3 ? h->sps_dev[sps_slot] : h->buf.maps[mode];
    const bool same = ms.bytes == bytes && (int64_t)shadow.size() == bytes && memcmp(shadow.data(), hb, bytes) == 0;
    if (!same) {
        if (bytes > 0) SD_HIP(h, hipMemcpyAsync(db, hb, bytes, hipMemcpyHostToDevice, h->st));
        shadow.assign(hb, hb + bytes);
    }
    ms.tokens = (int32_t*)(db + o_tok); ms.src = (int32_t*)(db + o_src); ms.pos = (int32_t*)(db + o_pos);
    ms.seq = (int32_t*)(db + o_seq); ms.kvl = (int32_t*)(db + o_kvl);
    ms.blk = (int32_t*)(db + o_blk); ms.kv_off = (int64_t*)(db + o_off); ms.tiles = (AttnTile*)(db + o_tiles);
    ms.order = (int32_t*)(db + o_order); ms.n_order = (int)n_order;
    ms.groups = (int32_t*)(db + o_groups); ms.n_groups = (int)n_groups; ms.group_tiles = group_tiles;
    ms.rows = (int)rows; ms.n_tiles = (int)n_tiles; ms.max_kv = max_kv; ms.kv_sum = kv_sum; ms.kv_rows = kv_rows;
    ms.head_row0 = (mode == 1 || mode == 3) ? 0 : (mode == 0 && batch == 1 ? len[0] : -1);   // target, autoregressive step: all rows; drafter: the block of a single sequence
    ms.regular = mode == 0 && batch == 1;
    ms.causal_base = batch == 1 && mode == 1 ? len[0] : (batch == 1 && mode == 3 ? len[0] + k : -1);
    ms.kv_row0 = (mode == 1 || mode == 3) && batch == 1 ? len[0] - 1 + k : -1;
    ms.grouped = grouped_order;
    ms.bytes = bytes;
    return SD_OK;
}

// Replay a launch sequence through a captured graph.  A sequence is launched eagerly the first time
// its key is seen and captured the second time (a generation loop changes its lengths every round and
// would otherwise pay for a capture it never replays).  `key` must
// identify everything that shapes the sequence: the call, batch, gamma, T, every sequence length
// and every pointer argument.  Falls back to eager launches when profiling is on, when the handle
// runs on the legacy default stream, or when capture is not possible.
template <typename F>
int replay(sd_handle* h, uint64_t key, F&& enqueue) {
    if (!h->use_graphs || h->prof.on || h->st == nullptr) {
        if (h->graph_failures > 0) ++h->graph_eager;
        return enqueue();
    }
    // A failed capture switches replay off for the handle (results stay correct, launches run eagerly); the
    // failure is kept in graph_error / sd_graph_stats so that a caller who times rounds can see it.
    auto give_up = [&](const char* what, hipError_t e) {
        h->use_graphs = false;
        ++h->graph_failures;
        h->graph_error = std::string(what) + ": " + hipGetErrorString(e);
        (void)hipGetLastError();
    };
    auto it = h->graphs.find(key);
    if (it == h->graphs.end()) {
        if (h->seen.insert(key).second) {
            if (h->seen.size() > 65536) h->seen.clear();
            return enqueue();
        }
        if (h->graphs.size() >= 256) {
            for (auto& g : h->graphs) (void)hipGraphExecDestroy(g.second);
            h->graphs.clear();
        }
        const hipError_t e0 = hipStreamBeginCapture(h->st, hipStreamCaptureModeThreadLocal);
        if (e0 != hipSuccess) {
            give_up("hipStreamBeginCapture", e0);
            ++h->graph_eager;
            return enqueue();
        }
        const int rc = enqueue();
        hipGraph_t graph = nullptr;
        const hipError_t e1 = hipStreamEndCapture(h->st, &graph);
        if (rc != SD_OK || e1 != hipSuccess || graph == nullptr) {
            if (graph) (void)hipGraphDestroy(graph);
            give_up(rc != SD_OK ? "launch sequence failed under capture" : "hipStreamEndCapture", e1);
            if (rc != SD_OK) return rc;
            ++h->graph_eager;
            return enqueue();
        }
        hipGraphExec_t exec = nullptr;
        const hipError_t e2 = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e2 != hipSuccess || exec == nullptr) {
            give_up("hipGraphInstantiate", e2);
            ++h->graph_eager;
            return enqueue();
        }
        it = h->graphs.emplace(key, exec).first;
    }
    SD_HIP(h, hipGraphLaunch(it->second, h->st));
    ++h->graph_replays;
    return SD_OK;
}

uint64_t shape_key(int call, int batch, int gamma, int T, const int32_t* len, const void* ptr) {
    uint64_t x = 1469598103934665603ull;
    auto mix = [&](uint64_t v) { x ^= v; x *= 1099511628211ull; };
    mix((uint64_t)call); mix((uint64_t)batch); mix((uint64_t)gamma); mix((uint64_t)T); mix((uint64_t)(uintptr_t)ptr);
    mix((uint64_t)(uint32_t)linear_mfma_get_variant()); mix((uint64_t)(uint32_t)linear_mfma_get_split());   // process-wide tuning hooks shape the launches too
    for (int b = 0; b < batch; ++b) mix((uint64_t)(uint32_t)len[b]);
    return x;
}

// Transformer layers over the rows described by the uploaded maps; residual stream in buf.h.
// The byte / flop figures passed to SD_LAUNCH are the algorithmic ones (operands read once,
// results written once).
int run_linear(sd_handle* h, int dt, const void* x, const void* w, const float* bias, void* y, int m, int n, int k,
               int ldy, int epi, const NormIn& ni = NormIn(), const NormOut& no = NormOut()) {
    const double ew = dt == SD_DTYPE_BF16 ? 2 : 4;
    const double out_b = epi == EPI_RESID ? 8.0 : (epi == EPI_F32 ? 4.0 : ew);
    const double bytes = ((double)m * k + (double)n * k) * ew + (double)m * n * (out_b + (no.gain ? 2.0 : 0.0));
    const char* name = "linear";
    SD_LAUNCH(h, name, bytes, 2.0 * m * n * k, launch_linear(dt, x, w, bias, y, m, n, k, ldy, epi, ni, no, h->buf.split, h->st, &name));
    return SD_OK;
}

// Transformer layers over the rows described by the uploaded maps; residual stream in buf.h.
//
// bf16 models: every normalisation in front of a contraction is folded into it (NormIn / NormOut).  Whoever
// writes the residual stream -- the embedding kernel, the attention-output and MLP-down contractions --
// also writes xn = bf16(h * gain of the next normalisation) and the partial row sums, so a layer is five
// launches (QKV, attention, attention-output, MLP-up, MLP-down) with no normalisation kernel.
// head_rows > 0: an LM head over head_rows rows follows; when those rows are one contiguous run the last residual
// epilogue also prepares the final normalisation for it (x = bf16(h gain_f), row sums), and run_head folds it.
int run_layers(sd_handle* h, const Model& m, const MapSet& rm, const float* temb, int head_rows = 0) {
    Buffers& B = h->buf;
    const sd_model_config& c = m.c;
    const int rows = rm.rows, d = c.d_model, dt = c.dtype;
    if (rows == 0) return SD_OK;
    const bool cached = !c.bidirectional;
    const int qkv_w = m.dq + 2 * m.dkv;
    const int up_w = c.arch == SD_ARCH_GPT2 ? c.d_ff : 2 * c.d_ff;
    const double ew = m.ew, rd = (double)rows * d;
    const bool ln = c.arch == SD_ARCH_GPT2;
    // all four contractions of a layer must be on the matrix-core path for the folded chain
    const bool fold = m.fold && linear_mfma_supported(dt, rows, qkv_w, d, qkv_w) && linear_mfma_supported(dt, rows, d, d, d) &&
                      linear_mfma_supported(dt, rows, up_w, d, up_w) && linear_mfma_supported(dt, rows, d, c.d_ff, d);
    const int parts_d = (d + 31) / 32;
    const bool head_fold = fold && head_rows > 0 && rm.head_row0 >= 0 && linear_mfma_supported(dt, head_rows, c.vocab, d, m.ld);
    h->head_folded = head_fold;
    int parts = 1;                      // partial row sums per row currently in buf.stats
    // r0: first row of the call (the row sums of row r sit at stats[r][parts][2], xn at xn[r][d])
    auto fold_in = [&](const float* u, int r0 = 0) {
        NormIn ni;
        ni.kind = ln ? 1 : 2; ni.stats = B.stats + (size_t)r0 * parts * 2; ni.parts = parts; ni.u = ln ? u : nullptr; ni.eps = c.norm_eps;
        return ni;
    };
    auto fold_out = [&](const float* gain, int r0 = 0) {
        NormOut no;
        no.gain = gain; no.xg = static_cast<char*>(B.xn) + (size_t)r0 * d * 2; no.stats = B.stats + (size_t)r0 * parts_d * 2;
        return no;
    };
    // Last layer of the drafter at batch 1: only the block's rows reach the LM head, and after the QKV contraction
    // (keys and values of every row are still needed) nothing else reads the prefix rows.  Attention, attention
    // output and MLP then run on the rows from t0 on (the 32-row tile that holds the block's first row).
    int t0 = 0;
    if (head_fold && !cached && rm.regular && rm.head_row0 >= 32) {
        const int cand = rm.head_row0 / 32 * 32, n = rows - cand;
        if (linear_mfma_supported(dt, n, d, d, d) && linear_mfma_supported(dt, n, up_w, d, up_w) && linear_mfma_supported(dt, n, d, c.d_ff, d)) t0 = cand;
    }
    int rc;
    SD_LAUNCH(h, "k_embed", rd * (4 + ew + (fold ? 2 : 0)), 0,
              launch_embed(dt, rm.src, rm.pos, rm.tokens, B.z, m.wte, m.wpe, temb, B.h, rows, d, fold ? m.L[0].ln1_g : nullptr, B.xn, B.stats, h->st));
    // The query rows of a single sequence sit at consecutive cache rows: the QKV contraction then writes its K and V
    // columns straight into the cache (few-row kernel, plain store epilogue) and no copy kernel runs.  With rotary
    // positions the same epilogue rotates q and k; the angles depend on the positions only: one table per forward.
    const bool kv_direct = fold && cached && rm.kv_row0 >= 0 && rows <= 64 && m.dq % 32 == 0 && m.dkv % 32 == 0 &&
                           (c.arch == SD_ARCH_GPT2 || ((m.dh == 64 || m.dh == 128) && qkv_w % 32 == 0));
    if (kv_direct && c.arch == SD_ARCH_LLAMA)
        SD_LAUNCH(h, "k_rope_table", 8.0 * rows * (m.dh / 2), 0, launch_rope_table(rm.pos, rows, m.dh, c.rope_theta, B.rope_cs, h->st));
    for (int i = 0; i < c.n_layer; ++i) {
        const Layer& l = m.L[i];
        const int64_t per_layer = cached ? (int64_t)h->max_batch * c.n_ctx * m.dkv * m.ew : 0;
        char* const kc = cached ? static_cast<char*>(m.kcache) + i * per_layer : nullptr;
        char* const vc = cached ? static_cast<char*>(m.vcache) + i * per_layer : nullptr;
        if (fold) {
            NormOut qkv_out;
            if (kv_direct) {
                qkv_out.y1 = kc + rm.kv_row0 * m.dkv * (int64_t)m.ew;
                qkv_out.y2 = vc + rm.kv_row0 * m.dkv * (int64_t)m.ew;
                qkv_out.c1 = m.dq; qkv_out.c2 = m.dq + m.dkv; qkv_out.ld12 = m.dkv;
                if (c.arch == SD_ARCH_LLAMA) { qkv_out.rope_cs = B.rope_cs; qkv_out.rope_cols = m.dq + m.dkv; qkv_out.rope_dh = m.dh; }
            }
            if ((rc = run_linear(h, dt, B.xn, l.w_qkv, ln ? l.fv_qkv : l.b_qkv, B.qkv, rows, qkv_w, d, qkv_w, EPI_STORE, fold_in(l.fu_qkv), qkv_out))) return rc;
        } else {
            SD_LAUNCH(h, "k_norm", rd * (4 + ew), 0, launch_norm(dt, B.h, nullptr, l.ln1_g, l.ln1_b, B.xn, rows, d, c.norm_eps, h->st));
            if ((rc = run_linear(h, dt, B.xn, l.w_qkv, l.b_qkv, B.qkv, rows, qkv_w, d, qkv_w, EPI_STORE))) return rc;
        }
        const bool rope_into_cache = c.arch == SD_ARCH_LLAMA && cached;     // one kernel for both
        if (c.arch == SD_ARCH_LLAMA && !rope_into_cache)
            SD_LAUNCH(h, "k_rope", 2.0 * rows * (m.dq + m.dkv) * ew, 0, launch_rope(dt, B.qkv, rm.pos, rows, c.n_head, c.n_kv_head, m.dh, c.rope_theta, h->st));
        // r0, nr: the rows everything after the QKV contraction runs on
        const int r0 = i + 1 == c.n_layer ? t0 : 0, nr = rows - r0;
        auto at = [&](void* p, int64_t width, int64_t esz) { return static_cast<void*>(static_cast<char*>(p) + (int64_t)r0 * width * esz); };
        AttnArgs a;
        a.q = at(B.qkv, qkv_w, m.ew); a.q_ld = qkv_w;
        a.kv_off = rm.kv_off; a.kv_len = rm.kvl;
        a.out = at(B.att, d, m.ew); a.out_ld = d;
        a.rows = nr; a.n_head = c.n_head; a.n_kv_head = c.n_kv_head; a.d_head = m.dh; a.max_kv = rm.max_kv;
        a.tiles = rm.tiles; a.n_tiles = r0 ? (nr + 31) / 32 : rm.n_tiles;
        a.regular = cached ? (rm.causal_base >= 0 ? 2 : 0) : (rm.regular ? 1 : 0);
        a.kv_base = rm.causal_base;
        if (rm.grouped && !r0) { a.order = rm.order; a.n_order = rm.n_order; }      // the plain order needs no table (and no load of it)
        if (!r0) { a.groups = rm.groups; a.n_groups = rm.n_groups; a.group_tiles = rm.group_tiles; }
        if (cached) {
            if (kv_direct) {
                // already in the cache
            } else if (rope_into_cache)
                SD_LAUNCH(h, "k_rope_kv_store", (2.0 * (m.dq + m.dkv) + 4.0 * m.dkv) * rows * ew, 0,
                          launch_rope_kv_store(dt, B.qkv, rm.seq, rm.pos, kc, vc, rows, c.n_head, c.n_kv_head, m.dh, c.rope_theta, c.n_ctx, h->st));
            else
                SD_LAUNCH(h, "k_kv_store", 4.0 * rows * m.dkv * ew, 0, launch_kv_store(dt, B.qkv, rm.seq, rm.pos, kc, vc, rows, c.n_head, c.n_kv_head, m.dh, c.n_ctx, h->st));
            a.k = kc; a.v = vc; a.kv_ld = m.dkv;
        } else {
            a.k = static_cast<char*>(B.qkv) + (int64_t)m.dq * m.ew;
            a.v = static_cast<char*>(B.qkv) + (int64_t)(m.dq + m.dkv) * m.ew;
            a.kv_ld = qkv_w;
        }
        const char* aname = "attention";
        SD_LAUNCH(h, aname, 2.0 * nr * d * ew + 2.0 * rm.kv_rows * m.dkv * ew, 4.0 * (r0 ? (double)nr * rm.max_kv : (double)rm.kv_sum) * d,
                  launch_attention(dt, a, h->st, &aname));
        // attention output: h += ..., and xn / row sums for the normalisation in front of the MLP
        if ((rc = run_linear(h, dt, at(B.att, d, m.ew), l.w_o, l.b_o, at(B.h, d, 4), nr, d, d, d, EPI_RESID, NormIn(), fold ? fold_out(l.ln2_g, r0) : NormOut()))) return rc;
        if (fold) parts = parts_d;
        if (!fold) SD_LAUNCH(h, "k_norm", rd * (4 + ew), 0, launch_norm(dt, B.h, nullptr, l.ln2_g, ln ? l.ln2_b : nullptr, B.xn, rows, d, c.norm_eps, h->st));
        const NormIn up_in = fold ? fold_in(l.fu_fc, r0) : NormIn();
        const float* up_bias = ln ? (fold ? l.fv_fc : l.b_fc) : nullptr;
        const void* down_x;
        if (ln) {
            if ((rc = run_linear(h, dt, at(B.xn, d, m.ew), l.w_fc, up_bias, at(B.mlp, up_w, m.ew), nr, up_w, d, up_w, EPI_GELU, up_in))) return rc;
            down_x = at(B.mlp, up_w, m.ew);
        } else {
            // Few rows against the long gate | up stream: the gating runs in the contraction's epilogue (gate and up tiles
            // of the same columns in one workgroup), gate / up never reach memory.  Otherwise contraction, then gating kernel.
            const bool gated = fold && nr <= 64 && up_w % 128 == 0;
            if (gated) {
                const double bytes = ((double)nr * d + (double)up_w * d) * ew + (double)nr * c.d_ff * ew;
                const char* name = "linear";
                SD_LAUNCH(h, name, bytes, 2.0 * nr * up_w * d,
                          launch_linear_stream(at(B.xn, d, m.ew), l.w_fc, nullptr, at(B.act, c.d_ff, m.ew), nr, up_w, d, c.d_ff, EPI_SWIGLU, up_in, NormOut(), h->buf.split, 0, h->st, &name));
            }
            if (!gated) {
                if ((rc = run_linear(h, dt, at(B.xn, d, m.ew), l.w_fc, up_bias, at(B.mlp, up_w, m.ew), nr, up_w, d, up_w, EPI_STORE, up_in))) return rc;
                SD_LAUNCH(h, "k_swiglu", 3.0 * nr * c.d_ff * ew, 0, launch_swiglu(dt, at(B.mlp, up_w, m.ew), at(B.act, c.d_ff, m.ew), nr, c.d_ff, h->st));
            }
            down_x = at(B.act, c.d_ff, m.ew);
        }
        // MLP down: h += ..., and xn / row sums for the first normalisation of the next layer
        const bool more = fold && i + 1 < c.n_layer;
        if ((rc = run_linear(h, dt, down_x, l.w_proj, ln ? l.b_proj : nullptr, at(B.h, d, 4), nr, d, c.d_ff, d, EPI_RESID, NormIn(),
                             more ? fold_out(m.L[i + 1].ln1_g) : (head_fold ? fold_out(m.lnf_g, r0) : NormOut())))) return rc;
    }
    return SD_OK;
}

// Final norm on selected rows + LM head -> fp32 logits [n_rows, ld].  idx: the rows (NULL: rows 0 .. n_rows - 1);
// row0: their first row when they are one contiguous run (MapSet::head_row0).
// tiles_out != NULL (temperature 0, where only the arg-maxima of the rows are needed): with up to 64 rows the head
// writes no logits at all but, per row and 32-column tile, the largest logit and its column -- values in `logits` as
// [n_rows][tiles], columns behind them as int32 [n_rows][tiles] -- and *tiles_out = tiles; otherwise *tiles_out = 0 and
// the logits are written as usual.
int run_head(sd_handle* h, const Model& m, const int32_t* idx, int row0, int n_rows, float* logits, int* tiles_out = nullptr) {
    Buffers& B = h->buf;
    const sd_model_config& c = m.c;
    const bool ln = c.arch == SD_ARCH_GPT2;
    const bool folded = h->head_folded && row0 >= 0;
    NormIn ni;
    const void* x = B.xf;
    if (folded) {
        // the last residual epilogue left x = bf16(h gain_f) and the row sums of every row: no normalisation kernel
        const int parts = (c.d_model + 31) / 32;
        ni.kind = ln ? 1 : 2; ni.stats = B.stats + (int64_t)row0 * parts * 2; ni.parts = parts; ni.u = ln ? m.fu_head : nullptr; ni.eps = c.norm_eps;
        x = static_cast<const char*>(B.xn) + (int64_t)row0 * c.d_model * 2;
    } else {
        SD_LAUNCH(h, "k_norm", (double)n_rows * c.d_model * (4 + m.ew), 0, launch_norm(c.dtype, B.h, idx, m.lnf_g, m.lnf_b, B.xf, n_rows, c.d_model, c.norm_eps, h->st));
    }
    const float* bias = folded && ln ? m.fv_head : nullptr;
    if (tiles_out) {
        *tiles_out = 0;
        if (n_rows <= 64 && linear_mfma_supported(c.dtype, n_rows, c.vocab, c.d_model, m.ld)) {
            const int tiles = (c.vocab + 31) / 32;
            NormOut no;
            no.am_v = logits;
            no.am_i = reinterpret_cast<int32_t*>(logits + (int64_t)n_rows * tiles);
            const double bytes = ((double)n_rows * c.d_model + (double)c.vocab * c.d_model) * m.ew + 8.0 * n_rows * tiles;
            const char* name = "linear";
            SD_LAUNCH(h, name, bytes, 2.0 * n_rows * c.vocab * c.d_model,
                      launch_linear_stream(x, m.w_head, bias, logits, n_rows, c.vocab, c.d_model, m.ld, EPI_ARGMAX, ni, no, h->buf.split, 0, h->st, &name));
            *tiles_out = tiles;
            return SD_OK;
        }
    }
    return run_linear(h, c.dtype, x, m.w_head, bias, logits, n_rows, c.vocab, c.d_model, m.ld, EPI_F32, ni);
}

int check_round_shapes(sd_handle* h, int batch, const int32_t* len, int gamma) {
    if (gamma <= 0 || gamma > h->gamma_max) return fail(h, SD_ERR_SHAPE, "gamma outside [1, gamma_max]");
    for (int b = 0; b < batch; ++b) {
        if (len[b] + gamma > h->drafter.c.n_ctx) return fail(h, SD_ERR_SHAPE, "prefix + gamma exceeds the drafter context");
        if (len[b] + gamma > h->target.c.n_ctx) return fail(h, SD_ERR_SHAPE, "prefix + gamma exceeds the target context");
    }
    return SD_OK;
}

int do_prefill(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int64_t n_tokens) {
    int rc = upload_rows(h, 2, batch, prefix, len, n_tokens, 0);
    if (rc) return rc;
    h->prof.phase = "prefill:";
    rc = run_layers(h, h->target, h->maps[2], nullptr);
    if (rc) return rc;
    int64_t off = 0;
    for (int b = 0; b < batch; ++b) {
        h->cached_len[b] = len[b] - 1;
        h->cached_fnv[b] = fnv_extend(kFnvBasis, prefix + off, len[b] - 1);
        h->cached_hash[b] = h->cached_fnv[b] ^ (uint64_t)(len[b] - 1);
        off += len[b];
    }
    h->pend_batch = 0;
    return SD_OK;
}

// Remember what a verification scored (the cache now also holds the K, V rows of prefix[L-1] and the draft).
void note_pending(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int gamma, const int32_t* draft, bool from_sps = false) {
    h->pend_batch = batch;
    h->pend_sps = from_sps;
    h->pend_gamma = gamma;
    h->pend_len.assign(len, len + batch);
    h->pend_tail.resize(batch);
    int64_t off = 0;
    for (int b = 0; b < batch; ++b) { off += len[b]; h->pend_tail[b] = prefix[off - 1]; }
    h->pend_draft.assign(draft, draft + (int64_t)batch * gamma);
}

bool cache_matches(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len) {
    int64_t off = 0;
    for (int b = 0; b < batch; ++b) {
        if (h->cached_len[b] != len[b] - 1 || h->cached_hash[b] != hash_tokens(prefix + off, len[b] - 1)) return false;
        off += len[b];
    }
    return true;
}

// Everything a draft needs on the device before its launches: row maps and the seed.
int prepare_draft(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int64_t n_tokens, int gamma,
                  uint64_t seed) {
    const int rc = upload_rows(h, 0, batch, prefix, len, n_tokens, gamma);
    if (rc) return rc;
    h->stage_seed[0] = seed;
    SD_HIP(h, hipMemcpyAsync(h->buf.seed, h->stage_seed, 8, hipMemcpyHostToDevice, h->st));
    return SD_OK;
}

// temb[j-1] for j = 1..T depends on the drafter's weights and on T only: built once per T (eagerly, outside any
// captured sequence) and kept in the workspace until a call asks for another T.
int ensure_timestep_table(sd_handle* h, int T) {
    if (h->temb_T == T) return SD_OK;
    const Model& m = h->drafter;
    h->prof.phase = "draft:";
    SD_LAUNCH(h, "k_timestep_matvec(x2)", 2.0 * m.c.d_model * m.c.d_model * m.ew, 4.0 * T * m.c.d_model * m.c.d_model,
              launch_timestep_embed(m.c.dtype, m.t_w1, m.t_b1, m.t_w2, m.t_b2, h->buf.temb_hidden, h->buf.temb, T, m.c.d_model, h->st));
    h->temb_T = T;
    return SD_OK;
}

// The T reverse-diffusion steps (launches only: capturable).  Leaves z (draft), q, qtok in the workspace.
// The timestep table is in place (ensure_timestep_table).
// z <- [MASK]^gamma
int enqueue_fill(sd_handle* h, int batch, int gamma) {
    h->prof.phase = "draft:";
    SD_LAUNCH(h, "k_fill_i32", 4.0 * batch * gamma, 0, launch_fill_i32(h->buf.z, batch * gamma, h->drafter.c.vocab, h->st));
    return SD_OK;
}

// Drafting step j of T: forward at t = j / T, LM head on the block rows, reveal + sample.
int enqueue_draft_step(sd_handle* h, int batch, int gamma, int T, int j) {
    Buffers& B = h->buf;
    const Model& m = h->drafter;
    const MapSet& rm = h->maps[0];
    h->prof.phase = "draft:";
    const SampleScratch ss = sampling_scratch(B.sample_scratch, (int)h->lim.rows_head, m.c.vocab);
    int rc = run_layers(h, m, rm, B.temb + (int64_t)(j - 1) * m.c.d_model, batch * gamma);
    if (rc) return rc;
    int tiles = 0;
    rc = run_head(h, m, rm.blk, rm.head_row0, batch * gamma, B.logits_d, h->greedy ? &tiles : nullptr);
    if (rc) return rc;
    if (h->greedy && tiles > 0) {
        const int rows = batch * gamma;
        SD_LAUNCH(h, "k_greedy_reveal_tiles", 8.0 * rows / T * tiles, 0,
                  launch_greedy_from_tiles(B.logits_d, reinterpret_cast<const int32_t*>(B.logits_d + (int64_t)rows * tiles), tiles, batch, gamma,
                                           m.c.vocab, j, -1, B.seed, B.z, B.qtok, h->st));
    } else if (h->greedy) {
        SD_LAUNCH(h, "unmask_greedy(k_chunk_argmax+k_greedy_reveal)", 1.0 * batch * gamma / T * m.ld * 4, 0,
                  launch_unmask_greedy(B.logits_d, batch, gamma, m.c.vocab, j, B.seed, B.z, B.qtok, ss, h->st));
    } else {
        SD_LAUNCH(h, "unmask_sample(k_row_stats+k_unmask_sample)", 3.0 * batch * gamma / T * m.ld * 4, 0,
                  launch_unmask_sample(B.logits_d, batch, gamma, m.c.vocab, j, B.seed, B.z, B.q, B.qtok, ss, h->st));
    }
    return SD_OK;
}

int enqueue_draft(sd_handle* h, int batch, int gamma, int T) {
    int rc = enqueue_fill(h, batch, gamma);
    for (int j = T; j >= 1 && !rc; --j) rc = enqueue_draft_step(h, batch, gamma, T, j);
    return rc;
}

// Which of the T drafting steps reveal at least one slot: needed[j] for j = 1 .. T; returns their number.  Whether a
// masked slot is revealed at step j is decided by its Philox draw alone (reveal_now), so the whole schedule is
// known before anything runs: slot (b, k) is revealed at the first j, counting down from T, whose draw says so.
// The logits of a step are read by the slots revealed at it and by nothing else.
int steps_that_reveal(int batch, int gamma, int T, uint64_t seed, std::vector<char>& needed) {
    needed.assign(T + 1, 0);
    for (int b = 0; b < batch; ++b)
        for (int k = 0; k < gamma; ++k)
            for (int j = T; j >= 1; --j)
                if (reveal_now(k, j, b, STREAM_DRAFT, seed)) { needed[j] = 1; break; }
    int n = 0;
    for (int j = 1; j <= T; ++j) n += needed[j];
    return n;
}

// The drafting part of a call, as graphs: one for all T steps, or -- leaving out the steps that reveal nothing -- one
// per step (every step has its own time embedding and counter, hence its own graph).  call: distinguishes the
// entry points in the graph keys.
int replay_draft(sd_handle* h, int call, int batch, int gamma, int T, const int32_t* prefix_len, uint64_t seed) {
    const int g = h->greedy ? 16 : 0;
    if (!h->skip_idle_steps) {
        h->steps_run = T;
        return replay(h, shape_key(call + g, batch, gamma, T, prefix_len, nullptr), [&] { return enqueue_draft(h, batch, gamma, T); });
    }
    std::vector<char> needed;
    h->steps_run = steps_that_reveal(batch, gamma, T, seed, needed);
    int rc = replay(h, shape_key(6 + g, batch, gamma, 0, prefix_len, nullptr), [&] { return enqueue_fill(h, batch, gamma); });
    for (int j = T; j >= 1 && !rc; --j)
        if (needed[j]) rc = replay(h, shape_key(7 + g, batch, gamma, T * 4096 + j, prefix_len, nullptr), [&] { return enqueue_draft_step(h, batch, gamma, T, j); });
    return rc;
}

// Prefill on demand and upload the maps of the gamma+1 query rows.
int prepare_target(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int64_t n_tokens, int gamma) {
    if (!cache_matches(h, batch, prefix, len)) {
        const int rc = do_prefill(h, batch, prefix, len, n_tokens);
        if (rc) return rc;
    }
    return upload_rows(h, 1, batch, prefix, len, n_tokens, gamma);
}

// Target forward over the gamma+1 query rows (draft tokens taken from buf.z) -> buf.logits_t (capturable).
// for_round: the acceptance step follows (at temperature 0 the head may then leave per-tile arg-maxima instead of logits);
// false for the parity hook, which wants the logits.
int enqueue_target(sd_handle* h, bool for_round = true) {
    const MapSet& rm = h->maps[1];
    h->prof.phase = "verify:";
    const int rc = run_layers(h, h->target, rm, nullptr, rm.rows);
    if (rc) return rc;
    h->target_tiles = 0;
    return run_head(h, h->target, nullptr, rm.head_row0, rm.rows, h->buf.logits_t, (h->greedy && for_round) ? &h->target_tiles : nullptr);
}

int enqueue_accept(sd_handle* h, int batch, int gamma, const float* q_dev) {
    h->prof.phase = "accept:";
    const SampleScratch ss = sampling_scratch(h->buf.sample_scratch, (int)h->lim.rows_head, h->target.c.vocab);
    if (h->greedy && h->target_tiles > 0) {
        const int rows = batch * (gamma + 1), tiles = h->target_tiles;
        SD_LAUNCH(h, "accept_greedy(k_row_argmax_tiles+k_greedy_accept_top)", 8.0 * rows * tiles, 0,
                  launch_accept_greedy_from_tiles(h->buf.logits_t, reinterpret_cast<const int32_t*>(h->buf.logits_t + (int64_t)rows * tiles), tiles,
                                                  h->buf.z, batch, gamma, ss.active, h->buf.n_acc, h->buf.tok, h->st));
        return SD_OK;
    }
    if (h->greedy) {
        SD_LAUNCH(h, "accept_greedy(k_chunk_argmax+k_greedy_accept)", (double)batch * (gamma + 1) * h->target.ld * 4, 0,
                  launch_accept_greedy(h->buf.logits_t, h->buf.z, batch, gamma, h->target.c.vocab, h->buf.n_acc, h->buf.tok, ss, h->st));
        return SD_OK;
    }
    SD_LAUNCH(h, "accept_resample(k_row_stats+k_accept_final)",
              ((double)batch * (gamma + 1) + 4.0 * batch) * h->target.ld * 4, 0,
              launch_accept_resample(h->buf.logits_t, q_dev, h->buf.z, batch, gamma, h->target.c.vocab, h->buf.seed,
                                     h->buf.n_acc, h->buf.tok, ss, h->st));
    return SD_OK;
}

int read_back(sd_handle* h, int32_t* dst, const int32_t* dev, int64_t n) {
    SD_HIP(h, hipMemcpyAsync(h->stage_out, dev, n * 4, hipMemcpyDeviceToHost, h->st));
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    memcpy(dst, h->stage_out, n * 4);
    return SD_OK;
}


// LayerNorms in front of QKV / MLP-up / LM head folded into those contractions: u = W g, v = W beta + bias into p
// (fold_floats(config) floats).  RMSNorm models need no vectors.
bool fold_model(Model& m, float* p, hipStream_t st) {
    m.fold = m.c.dtype == SD_DTYPE_BF16;
    if (!m.fold || m.c.arch != SD_ARCH_GPT2) return true;
    const int qkv = m.dq + 2 * m.dkv, F = m.c.d_ff, d = m.c.d_model;
    for (Layer& l : m.L) {
        l.fu_qkv = p; p += align_up(qkv, 64);
        l.fv_qkv = p; p += align_up(qkv, 64);
        l.fu_fc = p; p += align_up(F, 64);
        l.fv_fc = p; p += align_up(F, 64);
        if (launch_fold_norm(l.w_qkv, l.ln1_g, l.ln1_b, l.b_qkv, l.fu_qkv, l.fv_qkv, qkv, d, st) != hipSuccess ||
            launch_fold_norm(l.w_fc, l.ln2_g, l.ln2_b, l.b_fc, l.fu_fc, l.fv_fc, F, d, st) != hipSuccess)
            return false;
    }
    m.fu_head = p; p += align_up(m.c.vocab, 64);
    m.fv_head = p; p += align_up(m.c.vocab, 64);
    return launch_fold_norm(m.w_head, m.lnf_g, m.lnf_b, nullptr, m.fu_head, m.fv_head, m.c.vocab, d, st) == hipSuccess;
}

// ------------------------------------------------------------------------------------------
// standard speculative decoding: the autoregressive drafter
// ------------------------------------------------------------------------------------------
int64_t sps_step_map_bytes(int max_batch, int heads, int64_t prefix_cap) {
    const int64_t mb = max_batch;
    return align_up((prefix_cap + 6 * mb) * 4 + 64 + mb * 8 + mb * (int64_t)sizeof(AttnTile) + 64 + 2 * 8 * (mb + 1) * heads * 4, 256);
}

struct SpsCarve { void *kcache, *vcache; float* fold; std::vector<char*> maps; int64_t step_bytes; };

int64_t carve_sps(Arena& a, SpsCarve& out, const sd_model_config& c, const Limits& lim, int max_batch, int gamma_max) {
    const int64_t cache = (int64_t)c.n_layer * max_batch * c.n_ctx * c.n_kv_head * (c.d_model / c.n_head);
    const int ew = c.dtype == SD_DTYPE_BF16 ? 2 : 4;
    out.kcache = a.take<char>(cache, ew);
    out.vcache = a.take<char>(cache, ew);
    out.fold = a.take<float>(fold_floats(c));
    out.step_bytes = sps_step_map_bytes(max_batch, c.n_head, lim.prefix_cap);
    out.maps.clear();
    out.maps.push_back(a.take<char>(lim.map_bytes));                      // catch-up rows
    for (int k = 0; k < gamma_max; ++k) out.maps.push_back(a.take<char>(out.step_bytes));
    return a.off;
}

bool sps_config_ok(const sd_handle* h, const sd_model_config* c) {
    if (!config_ok(c) || c->bidirectional) return false;
    const sd_model_config& t = h->target.c;
    const int64_t qkv = (int64_t)c->d_model + 2 * (int64_t)c->n_kv_head * (c->d_model / c->n_head);
    const int64_t ff = (int64_t)c->d_ff * (c->arch == SD_ARCH_LLAMA ? 2 : 1);
    const int heads = std::max(h->target.c.n_head, h->drafter.c.n_head);
    return c->vocab == t.vocab && c->dtype == t.dtype && c->d_model <= h->lim.dmax && qkv <= h->lim.qkvmax && ff <= h->lim.ffmax &&
           (int64_t)h->max_batch * c->n_ctx <= h->lim.max_rows && c->n_head <= heads && h->gamma_max < c->n_ctx &&
           (c->arch != SD_ARCH_LLAMA || t.arch == SD_ARCH_LLAMA);            // the gated-MLP scratch exists for Llama-shaped targets only
}

// Bring the autoregressive drafter's cache up to tokens [0, L - 1) of every sequence: only the rows it does not hold yet
// (after a committed round: none, or the one row of the last accepted draft token).
int sps_catch_up(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int64_t n_tokens) {
    std::vector<int32_t> start(batch);
    bool any = false;
    int64_t off = 0;
    for (int b = 0; b < batch; ++b) {
        const int c = h->sps_cached_len[b];
        start[b] = (c >= 0 && c <= len[b] - 1 && fnv_extend(kFnvBasis, prefix + off, c) == h->sps_cached_fnv[b]) ? c : 0;
        any = any || start[b] < len[b] - 1;
        off += len[b];
    }
    if (!any) return SD_OK;
    int rc = upload_rows(h, 4, batch, prefix, len, n_tokens, 0, 0, start.data());
    if (rc) return rc;
    h->prof.phase = "prefill:";
    rc = run_layers(h, h->sps, h->sps_ms[0], nullptr);
    if (rc) return rc;
    off = 0;
    for (int b = 0; b < batch; ++b) {
        h->sps_cached_len[b] = len[b] - 1;
        h->sps_cached_fnv[b] = fnv_extend(kFnvBasis, prefix + off, len[b] - 1);
        off += len[b];
    }
    return SD_OK;
}

// Everything the gamma sequential steps need on the device before their launches: the drafter's cache, the row maps of
// every step, the seed.
int prepare_sps(sd_handle* h, int batch, const int32_t* prefix, const int32_t* len, int64_t n_tokens, int gamma, uint64_t seed) {
    for (int b = 0; b < batch; ++b)
        if (len[b] + gamma > h->sps.c.n_ctx) return fail(h, SD_ERR_SHAPE, "prefix + gamma exceeds the autoregressive drafter's context");
    int rc = sps_catch_up(h, batch, prefix, len, n_tokens);
    for (int k = 0; k < gamma && !rc; ++k) rc = upload_rows(h, 3, batch, prefix, len, k == 0 ? n_tokens : 0, gamma, k);
    if (rc) return rc;
    h->stage_seed[0] = seed;
    SD_HIP(h, hipMemcpyAsync(h->buf.seed, h->stage_seed, 8, hipMemcpyHostToDevice, h->st));
    return SD_OK;
}

// The gamma sequential drafter evaluations (launches only: capturable): step k scores the one new row of every
// sequence against the drafter's cache, and its token is sampled on the device before step k + 1 embeds it.
int enqueue_sps_draft(sd_handle* h, int batch, int gamma) {
    Buffers& B = h->buf;
    const Model& m = h->sps;
    h->prof.phase = "draft:";
    const SampleScratch ss = sampling_scratch(B.sample_scratch, (int)h->lim.rows_head, m.c.vocab);
    for (int k = 0; k < gamma; ++k) {
        const MapSet& rm = h->sps_ms[1 + k];
        int rc = run_layers(h, m, rm, nullptr, batch);
        if (rc) return rc;
        int tiles = 0;
        rc = run_head(h, m, nullptr, rm.head_row0, batch, B.logits_d, h->greedy ? &tiles : nullptr);
        if (rc) return rc;
        if (tiles > 0) {
            SD_LAUNCH(h, "k_greedy_reveal_tiles", 8.0 * batch * tiles, 0,
                      launch_greedy_from_tiles(B.logits_d, reinterpret_cast<const int32_t*>(B.logits_d + (int64_t)batch * tiles), tiles, batch, gamma,
                                               m.c.vocab, 0, k, B.seed, B.z, B.qtok, h->st));
            continue;
        }
        SD_LAUNCH(h, h->greedy ? "sps_sample(k_chunk_argmax+k_greedy_reveal)" : "sps_sample(k_row_stats+k_unmask_sample)",
                  (h->greedy ? 1.0 : 3.0) * batch * m.ld * 4, 0,
                  launch_sps_sample(B.logits_d, batch, gamma, m.c.vocab, k, B.seed, B.z, B.q, B.qtok, h->greedy, ss, h->st));
    }
    return SD_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// exported functions
// ------------------------------------------------------------------------------------------
static std::string g_create_error = "null handle";   // reported by sd_last_error(NULL)

// ------------------------------------------------------------------------------------------
// Scratch of the allocation-free entry point (sd_accept_resample_static): a fixed array in device memory instead of
// a caller workspace.  Every GPU holds its own copy at its own address; host code never uses the array's name as an
// address, only what hipGetSymbolAddress returned for the current device.
// ------------------------------------------------------------------------------------------
constexpr int64_t kStaticScratchBytes = 4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        g_create_error = "sd_accept_resample_static: no current HIP device";
        return SD_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            g_create_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
            return SD_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SD_OK;
}

__global__ void k_store_u64(uint64_t* p, uint64_t v) { *p = v; }
}  // namespace

extern "C" {

int32_t sd_vocab_pad(int32_t vocab) { return vocab_pad(vocab); }

int32_t sd_weight_count(const sd_model_config* cfg) {
    if (!config_ok(cfg)) return 0;
    std::vector<TensorDesc> t;
    int64_t total;
    build_layout(*cfg, t, total);
    return (int32_t)t.size();
}

int32_t sd_weight_desc(const sd_model_config* cfg, int32_t index, char* name, int32_t name_cap, int64_t* rows,
                       int64_t* cols, int32_t* elem_bytes, int64_t* offset) {
    if (!config_ok(cfg) || !name || name_cap <= 0 || !rows || !cols || !elem_bytes || !offset) return SD_ERR_ARG;
    std::vector<TensorDesc> t;
    int64_t total;
    build_layout(*cfg, t, total);
    if (index < 0 || index >= (int32_t)t.size()) return SD_ERR_ARG;
    const TensorDesc& d = t[index];
    if ((int32_t)d.name.size() + 1 > name_cap) return SD_ERR_ARG;
    memcpy(name, d.name.c_str(), d.name.size() + 1);
    *rows = d.rows; *cols = d.cols; *elem_bytes = d.elem; *offset = d.off;
    return SD_OK;
}

int64_t sd_weight_bytes(const sd_model_config* cfg) {
    if (!config_ok(cfg)) return 0;
    std::vector<TensorDesc> t;
    int64_t total;
    build_layout(*cfg, t, total);
    return total;
}

static bool pair_ok(const sd_model_config* t, const sd_model_config* d, int max_batch, int gamma_max) {
    return config_ok(t) && config_ok(d) && !t->bidirectional && d->bidirectional && t->vocab == d->vocab &&
           max_batch > 0 && max_batch <= 4096 && gamma_max > 0 && gamma_max <= 255 && gamma_max < t->n_ctx &&
           gamma_max < d->n_ctx;
}

int64_t sd_workspace_bytes(const sd_model_config* target, const sd_model_config* drafter, int32_t max_batch,
                           int32_t gamma_max) {
    if (!pair_ok(target, drafter, max_batch, gamma_max)) return 0;
    Arena a(nullptr);
    Buffers b;
    return carve(a, b, *target, *drafter, max_batch, gamma_max);
}

int32_t sd_create(const sd_model_config* target, const sd_model_config* drafter, const void* target_w,
                  const void* drafter_w, int32_t max_batch, int32_t gamma_max, void* workspace,
                  int64_t workspace_bytes, void* hip_stream, sd_handle** out) {
    if (!out) return SD_ERR_ARG;
    *out = nullptr;
    if (!target_w || !drafter_w || !workspace) return SD_ERR_ARG;
    if (!pair_ok(target, drafter, max_batch, gamma_max)) return SD_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(target_w) & 255) ||
        (reinterpret_cast<uintptr_t>(drafter_w) & 255))
        return SD_ERR_WORKSPACE;
    sd_handle* h = new (std::nothrow) sd_handle();
    if (!h) return SD_ERR_ARG;
    Arena a(workspace);
    const int64_t need = carve(a, h->buf, *target, *drafter, max_batch, gamma_max);
    if (need > workspace_bytes) { delete h; return SD_ERR_WORKSPACE; }
    if (!bind_model(h->target, *target, target_w) || !bind_model(h->drafter, *drafter, drafter_w)) { delete h; return SD_ERR_ARG; }
    if (launch_sampling_reset(sampling_scratch(h->buf.sample_scratch, (int)limits_of(*target, *drafter, max_batch, gamma_max).rows_head, target->vocab),
                             (int)limits_of(*target, *drafter, max_batch, gamma_max).rows_head, static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
        g_create_error = "clearing the sampling counters failed";
        delete h;
        return SD_ERR_HIP;
    }
    if (hipMemsetAsync(h->buf.split.base, 0, kSplitTicketBytes, static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
        g_create_error = "clearing the split-K tickets failed";
        delete h;
        return SD_ERR_HIP;
    }
    // Fold the LayerNorms in front of QKV and MLP-up into those contractions (bf16 models): u = W g, v = W beta + bias.
    if (!fold_model(h->target, h->buf.fold_t, static_cast<hipStream_t>(hip_stream)) ||
        !fold_model(h->drafter, h->buf.fold_d, static_cast<hipStream_t>(hip_stream))) {
        g_create_error = "launch of the norm-folding kernel failed";
        delete h;
        return SD_ERR_HIP;
    }
    if (hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
        g_create_error = "norm folding failed";
        delete h;
        return SD_ERR_HIP;
    }
    { void* fixed = nullptr; (void)static_scratch(&fixed); }     // set-up of the allocation-free entry point on this device (it retries by itself if this failed)
    h->target.kcache = h->buf.kcache;
    h->target.vcache = h->buf.vcache;
    h->lim = limits_of(*target, *drafter, max_batch, gamma_max);
    h->max_batch = max_batch;
    h->gamma_max = gamma_max;
    h->st = static_cast<hipStream_t>(hip_stream);
    h->cached_len.assign(max_batch, -1);
    h->cached_hash.assign(max_batch, 0);
    h->cached_fnv.assign(max_batch, 0);
    const int64_t n_out = (int64_t)max_batch * (gamma_max + 2) + 16;
    struct { void** p; int64_t bytes; } pinned[] = {
        {reinterpret_cast<void**>(&h->stage_maps[0]), h->lim.map_bytes},
        {reinterpret_cast<void**>(&h->stage_maps[1]), h->lim.map_bytes},
        {reinterpret_cast<void**>(&h->stage_maps[2]), h->lim.map_bytes},
        {reinterpret_cast<void**>(&h->stage_seed), 64},
        {reinterpret_cast<void**>(&h->stage_z), n_out * 4},
        {reinterpret_cast<void**>(&h->stage_out), n_out * 4},
        {reinterpret_cast<void**>(&h->stage_f), n_out * 4}};
    for (auto& a : pinned) {
        const hipError_t e = hipHostMalloc(a.p, a.bytes, hipHostMallocDefault);
        if (e != hipSuccess) {
            g_create_error = std::string("hipHostMalloc(") + std::to_string(a.bytes) + "): " + hipGetErrorString(e);
            sd_destroy(h);
            return SD_ERR_HIP;
        }
    }
    *out = h;
    return SD_OK;
}

void sd_destroy(sd_handle* h) {
    if (!h) return;
    for (hipEvent_t e : h->prof.events) (void)hipEventDestroy(e);
    for (auto& g : h->graphs) (void)hipGraphExecDestroy(g.second);
    for (int i = 0; i < 3; ++i)
        if (h->stage_maps[i]) (void)hipHostFree(h->stage_maps[i]);
    if (h->stage_seed) (void)hipHostFree(h->stage_seed);
    if (h->stage_z) (void)hipHostFree(h->stage_z);
    if (h->stage_out) (void)hipHostFree(h->stage_out);
    if (h->stage_f) (void)hipHostFree(h->stage_f);
    for (char* p : h->sps_stage) if (p) (void)hipHostFree(p);
    delete h;
}

const char* sd_last_error(const sd_handle* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int32_t sd_prefill(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    for (int b = 0; b < batch; ++b)
        if (prefix_len[b] > h->target.c.n_ctx) return fail(h, SD_ERR_SHAPE, "prefix exceeds the target context");
    rc = do_prefill(h, batch, prefix, prefix_len, n);
    if (rc) return rc;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    return SD_OK;
}

int32_t sd_draft(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len, int32_t gamma,
                 int32_t T, uint64_t seed, int32_t* draft_out, float* qtok_out, const float** q_dev_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->drafter.c.vocab : 0, &n);
    if (rc) return rc;
    if (!draft_out) return fail(h, SD_ERR_ARG, "draft_out is null");
    if (T <= 0 || T > kMaxSteps) return fail(h, SD_ERR_SHAPE, "T outside [1, 256]");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    rc = prepare_draft(h, batch, prefix, prefix_len, n, gamma, seed);
    if (rc) return rc;
    rc = ensure_timestep_table(h, T);
    if (rc) return rc;
    rc = replay_draft(h, 1, batch, gamma, T, prefix_len, seed);
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    SD_HIP(h, hipMemcpyAsync(h->stage_out, h->buf.z, cnt * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(h->stage_f, h->buf.qtok, cnt * 4, hipMemcpyDeviceToHost, h->st));
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    memcpy(draft_out, h->stage_out, cnt * 4);
    if (qtok_out) memcpy(qtok_out, h->stage_f, cnt * 4);
    if (q_dev_out) *q_dev_out = h->greedy ? nullptr : h->buf.q;      // temperature 0 produces no q
    h->last_draft_sps = false;
    return SD_OK;
}

int32_t sd_verify(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len, int32_t gamma,
                  const int32_t* draft, const float* q_dev, uint64_t seed, int32_t* n_accepted_out,
                  int32_t* token_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!draft || (!q_dev && !h->greedy) || !n_accepted_out || !token_out) return fail(h, SD_ERR_ARG, "null argument");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    for (int64_t i = 0; i < cnt; ++i)
        if (draft[i] < 0 || draft[i] >= h->target.c.vocab) return fail(h, SD_ERR_TOKEN, "draft token outside the vocabulary");
    memcpy(h->stage_z, draft, cnt * 4);
    SD_HIP(h, hipMemcpyAsync(h->buf.z, h->stage_z, cnt * 4, hipMemcpyHostToDevice, h->st));
    h->stage_seed[0] = seed;
    SD_HIP(h, hipMemcpyAsync(h->buf.seed, h->stage_seed, 8, hipMemcpyHostToDevice, h->st));
    rc = prepare_target(h, batch, prefix, prefix_len, n, gamma);
    if (rc) return rc;
    rc = replay(h, shape_key(2 + (h->greedy ? 16 : 0), batch, gamma, 0, prefix_len, q_dev), [&] {
        const int r2 = enqueue_target(h);
        return r2 ? r2 : enqueue_accept(h, batch, gamma, q_dev);
    });
    if (rc) return rc;
    rc = read_back(h, n_accepted_out, h->buf.n_acc, batch);
    if (rc) return rc;
    rc = read_back(h, token_out, h->buf.tok, batch);
    if (rc) return rc;
    note_pending(h, batch, prefix, prefix_len, gamma, draft, h->last_draft_sps);
    return SD_OK;
}

int32_t sd_round(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len, int32_t gamma,
                 int32_t T, uint64_t seed, int32_t* draft_out, int32_t* n_accepted_out, int32_t* token_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!draft_out || !n_accepted_out || !token_out) return fail(h, SD_ERR_ARG, "null argument");
    if (T <= 0 || T > kMaxSteps) return fail(h, SD_ERR_SHAPE, "T outside [1, 256]");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    rc = prepare_draft(h, batch, prefix, prefix_len, n, gamma, seed);
    if (rc) return rc;
    rc = prepare_target(h, batch, prefix, prefix_len, n, gamma);
    if (rc) return rc;
    rc = ensure_timestep_table(h, T);
    if (rc) return rc;
    if (!h->skip_idle_steps) {
        h->steps_run = T;
        rc = replay(h, shape_key(3 + (h->greedy ? 16 : 0), batch, gamma, T, prefix_len, nullptr), [&] {
            int r2 = enqueue_draft(h, batch, gamma, T);
            if (!r2) r2 = enqueue_target(h);
            return r2 ? r2 : enqueue_accept(h, batch, gamma, h->buf.q);
        });
    } else {
        rc = replay_draft(h, 3, batch, gamma, T, prefix_len, seed);
        if (!rc)
            rc = replay(h, shape_key(8 + (h->greedy ? 16 : 0), batch, gamma, 0, prefix_len, nullptr), [&] {
                const int r2 = enqueue_target(h);
                return r2 ? r2 : enqueue_accept(h, batch, gamma, h->buf.q);
            });
    }
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    int32_t* so = h->stage_out;
    SD_HIP(h, hipMemcpyAsync(so, h->buf.z, cnt * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(so + cnt, h->buf.n_acc, batch * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(so + cnt + batch, h->buf.tok, batch * 4, hipMemcpyDeviceToHost, h->st));
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    memcpy(draft_out, so, cnt * 4);
    memcpy(n_accepted_out, so + cnt, batch * 4);
    memcpy(token_out, so + cnt + batch, batch * 4);
    note_pending(h, batch, prefix, prefix_len, gamma, draft_out);
    return SD_OK;
}

int32_t sd_commit(sd_handle* h, int32_t batch, const int32_t* n_accepted) {
    if (!h) return SD_ERR_ARG;
    if (!n_accepted) return fail(h, SD_ERR_ARG, "n_accepted is null");
    if (h->pend_batch == 0 || batch != h->pend_batch) return fail(h, SD_ERR_STATE, "no verification of this batch to commit");
    for (int b = 0; b < batch; ++b)
        if (n_accepted[b] < 0 || n_accepted[b] > h->pend_gamma) return fail(h, SD_ERR_ARG, "n_accepted outside [0, gamma]");
    for (int b = 0; b < batch; ++b) {
        if (h->cached_len[b] != h->pend_len[b] - 1) return fail(h, SD_ERR_STATE, "KV cache no longer matches the verified prefix");
        uint64_t x = fnv_extend(h->cached_fnv[b], &h->pend_tail[b], 1);
        x = fnv_extend(x, h->pend_draft.data() + (int64_t)b * h->pend_gamma, n_accepted[b]);
        h->cached_fnv[b] = x;
        h->cached_len[b] = h->pend_len[b] + n_accepted[b];
        h->cached_hash[b] = x ^ (uint64_t)h->cached_len[b];
    }
    if (h->has_sps && h->pend_sps) {
        // the autoregressive drafter's cache holds the rows of the last prefix token and of draft[0 .. gamma - 1)
        for (int b = 0; b < batch; ++b) {
            if (h->sps_cached_len[b] != h->pend_len[b] - 1) continue;                // not the string this round extended
            const int keep = std::min(n_accepted[b], h->pend_gamma - 1);
            uint64_t x = fnv_extend(h->sps_cached_fnv[b], &h->pend_tail[b], 1);
            x = fnv_extend(x, h->pend_draft.data() + (int64_t)b * h->pend_gamma, keep);
            h->sps_cached_fnv[b] = x;
            h->sps_cached_len[b] = h->pend_len[b] + keep;
        }
    }
    h->pend_batch = 0;
    return SD_OK;
}

int32_t sd_set_step_skipping(sd_handle* h, int32_t enable) {
    if (!h) return SD_ERR_ARG;
    h->skip_idle_steps = enable != 0;
    return SD_OK;
}

int32_t sd_steps_run(const sd_handle* h) { return h ? h->steps_run : -1; }

int32_t sd_set_greedy(sd_handle* h, int32_t enable) {
    if (!h) return SD_ERR_ARG;
    h->greedy = enable != 0;
    return SD_OK;
}

int32_t sd_drafter_logits(sd_handle* h, int32_t batch, const int32_t* tokens, const int32_t* seq_len, int32_t gamma,
                          int32_t step, int32_t T, const float** logits_dev_out) {
    int64_t n;
    int rc = check_batch(h, batch, tokens, seq_len, h ? h->drafter.c.vocab + 1 : 0, &n);
    if (rc) return rc;
    if (!logits_dev_out) return fail(h, SD_ERR_ARG, "logits_dev_out is null");
    if (T <= 0 || T > kMaxSteps || step < 1 || step > T) return fail(h, SD_ERR_SHAPE, "step / T out of range");
    if (gamma <= 0 || gamma > h->gamma_max) return fail(h, SD_ERR_SHAPE, "gamma outside [1, gamma_max]");
    std::vector<int32_t> plen(batch);
    for (int b = 0; b < batch; ++b) {
        if (seq_len[b] <= gamma || seq_len[b] > h->drafter.c.n_ctx)
            return fail(h, SD_ERR_SHAPE, "sequence must hold a prefix and gamma slots within the drafter context");
        plen[b] = seq_len[b] - gamma;
    }
    // Rows are described as prefix + gamma block slots; the block tokens are copied into z.
    std::vector<int32_t> pre, blk((size_t)batch * gamma);
    pre.reserve(n);
    int64_t off = 0;
    for (int b = 0; b < batch; ++b) {
        pre.insert(pre.end(), tokens + off, tokens + off + plen[b]);
        for (int k = 0; k < gamma; ++k) blk[(size_t)b * gamma + k] = tokens[off + plen[b] + k];
        off += seq_len[b];
    }
    rc = upload_rows(h, 0, batch, pre.data(), plen.data(), (int64_t)pre.size(), gamma);
    if (rc) return rc;
    memcpy(h->stage_z, blk.data(), blk.size() * 4);
    SD_HIP(h, hipMemcpyAsync(h->buf.z, h->stage_z, blk.size() * 4, hipMemcpyHostToDevice, h->st));
    const Model& m = h->drafter;
    rc = ensure_timestep_table(h, T);
    if (rc) return rc;
    rc = run_layers(h, m, h->maps[0], h->buf.temb + (int64_t)(step - 1) * m.c.d_model, batch * gamma);
    if (rc) return rc;
    rc = run_head(h, m, h->maps[0].blk, h->maps[0].head_row0, batch * gamma, h->buf.logits_d);
    if (rc) return rc;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    *logits_dev_out = h->buf.logits_d;
    return SD_OK;
}

int32_t sd_target_logits(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len,
                         int32_t gamma, const int32_t* draft, const float** logits_dev_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!draft || !logits_dev_out) return fail(h, SD_ERR_ARG, "null argument");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    for (int64_t i = 0; i < cnt; ++i)
        if (draft[i] < 0 || draft[i] >= h->target.c.vocab) return fail(h, SD_ERR_TOKEN, "draft token outside the vocabulary");
    memcpy(h->stage_z, draft, cnt * 4);
    SD_HIP(h, hipMemcpyAsync(h->buf.z, h->stage_z, cnt * 4, hipMemcpyHostToDevice, h->st));
    rc = prepare_target(h, batch, prefix, prefix_len, n, gamma);
    if (rc) return rc;
    rc = enqueue_target(h, false);
    if (rc) return rc;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    *logits_dev_out = h->buf.logits_t;
    return SD_OK;
}

int64_t sd_sps_workspace_bytes(const sd_handle* h, const sd_model_config* sps) {
    if (!h || !sps_config_ok(h, sps)) return 0;
    Arena a(nullptr);
    SpsCarve c;
    return carve_sps(a, c, *sps, h->lim, h->max_batch, h->gamma_max);
}

int32_t sd_sps_attach(sd_handle* h, const sd_model_config* sps, const void* sps_w, void* workspace, int64_t workspace_bytes) {
    if (!h) return SD_ERR_ARG;
    if (!sps || !sps_w || !workspace) return fail(h, SD_ERR_ARG, "null argument");
    if (h->has_sps) return fail(h, SD_ERR_STATE, "an autoregressive drafter is already attached");
    if (!sps_config_ok(h, sps)) return fail(h, SD_ERR_ARG, "autoregressive drafter must be causal, share vocabulary and storage type with the target and fit the handle's activation buffers");
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) || (reinterpret_cast<uintptr_t>(sps_w) & 255)) return fail(h, SD_ERR_WORKSPACE, "misaligned buffer");
    Arena a(workspace);
    SpsCarve c;
    if (carve_sps(a, c, *sps, h->lim, h->max_batch, h->gamma_max) > workspace_bytes) return fail(h, SD_ERR_WORKSPACE, "workspace too small");
    if (!bind_model(h->sps, *sps, sps_w)) return fail(h, SD_ERR_ARG, "weight layout");
    h->sps.kcache = c.kcache;
    h->sps.vcache = c.vcache;
    if (!fold_model(h->sps, c.fold, h->st)) return fail(h, SD_ERR_HIP, "launch of the norm-folding kernel failed");
    SD_HIP(h, hipStreamSynchronize(h->st));
    h->sps_map_cap = c.step_bytes;
    h->sps_dev = c.maps;
    h->sps_stage.assign(c.maps.size(), nullptr);
    for (size_t i = 0; i < c.maps.size(); ++i) {
        const hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&h->sps_stage[i]), i == 0 ? h->lim.map_bytes : c.step_bytes, hipHostMallocDefault);
        if (e != hipSuccess) {
            for (char* p : h->sps_stage) if (p) (void)hipHostFree(p);
            h->sps_stage.clear();
            h->err = std::string("hipHostMalloc: ") + hipGetErrorString(e);
            return SD_ERR_HIP;
        }
    }
    h->sps_ms.assign(c.maps.size(), MapSet());
    h->sps_shadow.assign(c.maps.size(), std::vector<char>());
    h->sps_cached_len.assign(h->max_batch, -1);
    h->sps_cached_fnv.assign(h->max_batch, 0);
    h->has_sps = true;
    return SD_OK;
}

int32_t sd_sps_draft(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len, int32_t gamma,
                     uint64_t seed, int32_t* draft_out, float* qtok_out, const float** q_dev_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!h->has_sps) return fail(h, SD_ERR_STATE, "no autoregressive drafter attached (sd_sps_attach)");
    if (!draft_out) return fail(h, SD_ERR_ARG, "draft_out is null");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    rc = prepare_sps(h, batch, prefix, prefix_len, n, gamma, seed);
    if (rc) return rc;
    h->steps_run = gamma;
    rc = replay(h, shape_key(9 + (h->greedy ? 16 : 0), batch, gamma, 0, prefix_len, nullptr), [&] { return enqueue_sps_draft(h, batch, gamma); });
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    SD_HIP(h, hipMemcpyAsync(h->stage_out, h->buf.z, cnt * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(h->stage_f, h->buf.qtok, cnt * 4, hipMemcpyDeviceToHost, h->st));
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    memcpy(draft_out, h->stage_out, cnt * 4);
    if (qtok_out) memcpy(qtok_out, h->stage_f, cnt * 4);
    if (q_dev_out) *q_dev_out = h->greedy ? nullptr : h->buf.q;
    h->last_draft_sps = true;
    return SD_OK;
}

int32_t sd_sps_round(sd_handle* h, int32_t batch, const int32_t* prefix, const int32_t* prefix_len, int32_t gamma,
                     uint64_t seed, int32_t* draft_out, int32_t* n_accepted_out, int32_t* token_out) {
    int64_t n;
    int rc = check_batch(h, batch, prefix, prefix_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!h->has_sps) return fail(h, SD_ERR_STATE, "no autoregressive drafter attached (sd_sps_attach)");
    if (!draft_out || !n_accepted_out || !token_out) return fail(h, SD_ERR_ARG, "null argument");
    rc = check_round_shapes(h, batch, prefix_len, gamma);
    if (rc) return rc;
    rc = prepare_sps(h, batch, prefix, prefix_len, n, gamma, seed);
    if (rc) return rc;
    rc = prepare_target(h, batch, prefix, prefix_len, n, gamma);
    if (rc) return rc;
    h->steps_run = gamma;
    rc = replay(h, shape_key(10 + (h->greedy ? 16 : 0), batch, gamma, 0, prefix_len, nullptr), [&] {
        int r2 = enqueue_sps_draft(h, batch, gamma);
        if (!r2) r2 = enqueue_target(h);
        return r2 ? r2 : enqueue_accept(h, batch, gamma, h->buf.q);
    });
    if (rc) return rc;
    const int64_t cnt = (int64_t)batch * gamma;
    int32_t* so = h->stage_out;
    SD_HIP(h, hipMemcpyAsync(so, h->buf.z, cnt * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(so + cnt, h->buf.n_acc, batch * 4, hipMemcpyDeviceToHost, h->st));
    SD_HIP(h, hipMemcpyAsync(so + cnt + batch, h->buf.tok, batch * 4, hipMemcpyDeviceToHost, h->st));
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    memcpy(draft_out, so, cnt * 4);
    memcpy(n_accepted_out, so + cnt, batch * 4);
    memcpy(token_out, so + cnt + batch, batch * 4);
    note_pending(h, batch, prefix, prefix_len, gamma, draft_out, true);
    return SD_OK;
}

int32_t sd_sps_logits(sd_handle* h, int32_t batch, const int32_t* tokens, const int32_t* seq_len, const float** logits_dev_out) {
    int64_t n;
    int rc = check_batch(h, batch, tokens, seq_len, h ? h->target.c.vocab : 0, &n);
    if (rc) return rc;
    if (!h->has_sps) return fail(h, SD_ERR_STATE, "no autoregressive drafter attached (sd_sps_attach)");
    if (!logits_dev_out) return fail(h, SD_ERR_ARG, "logits_dev_out is null");
    for (int b = 0; b < batch; ++b)
        if (seq_len[b] > h->sps.c.n_ctx) return fail(h, SD_ERR_SHAPE, "sequence exceeds the autoregressive drafter's context");
    rc = sps_catch_up(h, batch, tokens, seq_len, n);
    if (!rc) rc = upload_rows(h, 3, batch, tokens, seq_len, n, 1, 0);
    if (rc) return rc;
    h->prof.phase = "";
    rc = run_layers(h, h->sps, h->sps_ms[1], nullptr, batch);
    if (!rc) rc = run_head(h, h->sps, nullptr, h->sps_ms[1].head_row0, batch, h->buf.logits_d);
    if (rc) return rc;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    *logits_dev_out = h->buf.logits_d;
    return SD_OK;
}

int32_t sd_set_graph_replay(sd_handle* h, int32_t enable) {
    if (!h) return SD_ERR_ARG;
    h->use_graphs = enable != 0;
    return SD_OK;
}

int32_t sd_graph_stats(const sd_handle* h, int64_t* replays, int64_t* eager_after_failure, int32_t* failures,
                       int32_t* captured) {
    if (!h) return SD_ERR_ARG;
    if (replays) *replays = h->graph_replays;
    if (eager_after_failure) *eager_after_failure = h->graph_eager;
    if (failures) *failures = h->graph_failures;
    if (captured) *captured = (int32_t)h->graphs.size();
    return SD_OK;
}

const char* sd_graph_error(const sd_handle* h) { return h ? h->graph_error.c_str() : ""; }

int32_t sd_profile_begin(sd_handle* h) {
    if (!h) return SD_ERR_ARG;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    h->prof.entries.clear();
    h->prof.on = true;
    return SD_OK;
}

int32_t sd_profile_end(sd_handle* h) {
    if (!h) return SD_ERR_ARG;
    { const int rc_ = sync_stream(h); if (rc_) return rc_; }
    h->prof.on = false;
    return (int32_t)SD_OK;
}

int32_t sd_profile_count(const sd_handle* h) { return h ? (int32_t)h->prof.entries.size() : 0; }

int32_t sd_profile_entry(const sd_handle* h, int32_t index, char* name, int32_t name_cap, int64_t* launches,
                         double* total_ms, double* bytes, double* flops) {
    if (!h || !name || name_cap <= 0 || !launches || !total_ms || !bytes || !flops) return SD_ERR_ARG;
    if (index < 0 || index >= (int32_t)h->prof.entries.size()) return SD_ERR_ARG;
    const ProfEntry& e = h->prof.entries[index];
    const size_t n = e.name.size() < (size_t)name_cap - 1 ? e.name.size() : (size_t)name_cap - 1;
    memcpy(name, e.name.c_str(), n);
    name[n] = 0;
    *launches = e.launches; *total_ms = e.ms; *bytes = e.bytes; *flops = e.flops;
    return SD_OK;
}

int64_t sd_sampling_scratch_bytes(int32_t rows, int32_t vocab) { return sampling_scratch_bytes(rows, vocab); }

int32_t sd_unmask_sample(const float* logits, int32_t batch, int32_t gamma, int32_t vocab, int32_t step,
                         uint64_t seed, int32_t* z, float* q, float* qtok, void* scratch, int64_t scratch_bytes,
                         void* hip_stream) {
    if (!logits || !z || !q || !qtok || !scratch) return SD_ERR_ARG;
    if (batch <= 0 || gamma <= 0 || vocab <= 0 || step < 1 || vocab > kChunk * 512) return SD_ERR_SHAPE;
    if (scratch_bytes < sampling_scratch_bytes(batch * (gamma + 1), vocab) || (reinterpret_cast<uintptr_t>(scratch) & 255))
        return SD_ERR_WORKSPACE;
    const SampleScratch ss = sampling_scratch(scratch, batch * (gamma + 1), vocab);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(ss.seed, &seed, 8, hipMemcpyHostToDevice, st) != hipSuccess) return SD_ERR_HIP;   // pageable source: staged before return
    return launch_unmask_sample(logits, batch, gamma, vocab, step, ss.seed, z, q, qtok, ss, st) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int32_t sd_accept_resample(const float* p_logits, const float* q, const int32_t* draft, int32_t batch, int32_t gamma,
                           int32_t vocab, uint64_t seed, int32_t* n_accepted, int32_t* token, void* scratch,
                           int64_t scratch_bytes, void* hip_stream) {
    if (!p_logits || !q || !draft || !n_accepted || !token || !scratch) return SD_ERR_ARG;
    if (batch <= 0 || gamma <= 0 || vocab <= 0 || vocab > kChunk * 512 || gamma > 4095) return SD_ERR_SHAPE;
    if (scratch_bytes < sampling_scratch_bytes(batch * (gamma + 1), vocab) || (reinterpret_cast<uintptr_t>(scratch) & 255))
        return SD_ERR_WORKSPACE;
    const SampleScratch ss = sampling_scratch(scratch, batch * (gamma + 1), vocab);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(ss.seed, &seed, 8, hipMemcpyHostToDevice, st) != hipSuccess) return SD_ERR_HIP;   // pageable source: staged before return
    if (launch_sampling_reset(ss, batch * (gamma + 1), st) != hipSuccess) return SD_ERR_HIP;             // caller memory of unknown content
    return launch_accept_resample(p_logits, q, draft, batch, gamma, vocab, ss.seed, n_accepted, token, ss, st) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int64_t sd_static_scratch_bytes(void) { return kStaticScratchBytes; }

int32_t sd_accept_resample_static(const float* p_logits, const float* q, const int32_t* draft, int32_t batch, int32_t gamma,
                                  int32_t vocab, uint64_t seed, int32_t* n_accepted, int32_t* token, void* hip_stream) {
    if (!p_logits || !q || !draft || !n_accepted || !token) return SD_ERR_ARG;
    if (batch <= 0 || gamma <= 0 || vocab <= 0 || vocab > kChunk * 512 || gamma > 4095) return SD_ERR_SHAPE;
    const int64_t rows = (int64_t)batch * (gamma + 1);
    if (rows > (1 << 20) || sampling_scratch_bytes((int)rows, vocab) > kStaticScratchBytes) {
        g_create_error = "sd_accept_resample_static: batch * (gamma + 1) rows of this vocabulary need " +
                         std::to_string(rows > (1 << 20) ? -1 : sampling_scratch_bytes((int)rows, vocab)) + " bytes of scratch, the fixed buffer holds " +
                         std::to_string(kStaticScratchBytes) + "; use sd_accept_resample with a workspace";
        return SD_ERR_WORKSPACE;
    }
    void* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc) return rc;
    const SampleScratch ss = sampling_scratch(base, (int)rows, vocab);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // The arrival counters must start at zero (the array keeps whatever the last call, possibly an interrupted one, left):
    // cleared by a kernel.  Everything else -- partials, row statistics, the seed slot -- is written by this call before
    // it is read.  The seed travels as a kernel argument (no staging copy).
    if (launch_sampling_reset(ss, (int)rows, st) != hipSuccess) return SD_ERR_HIP;
    launch_kernel(k_store_u64, dim3(1), dim3(1), 0, st, ss.seed, seed);
    if (hipGetLastError() != hipSuccess) return SD_ERR_HIP;
    return launch_accept_resample(p_logits, q, draft, batch, gamma, vocab, ss.seed, n_accepted, token, ss, st) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int64_t sd_norm_linear_scratch_floats(int32_t m, int32_t n, int32_t k) {
    return 2 * (int64_t)align_up(n, 64) + 2 * (int64_t)align_up(m, 64) + ((int64_t)m * k + 1) / 2 + 64;
}

int32_t sd_norm_linear(int32_t norm_kind, const float* h, const void* w, const float* gain, const float* beta,
                       const float* bias, void* y, int32_t m, int32_t n, int32_t k, int32_t ldy, int32_t epilogue,
                       float eps, float* fold_scratch, void* split_workspace, int64_t split_workspace_bytes,
                       void* hip_stream) {
    if (!h || !w || !gain || !y || !fold_scratch) return SD_ERR_ARG;
    if (split_workspace && ((reinterpret_cast<uintptr_t>(split_workspace) & 255) || split_workspace_bytes <= kSplitTicketBytes))
        return SD_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(fold_scratch) & 255) return SD_ERR_WORKSPACE;
    const SplitWorkspace ws{split_workspace, split_workspace ? split_workspace_bytes : 0};
    if (norm_kind != 1 && norm_kind != 2) return SD_ERR_ARG;
    if (m <= 0 || n <= 0 || k <= 0 || ldy < n || epilogue < 0 || epilogue > 3 || epilogue == EPI_RESID) return SD_ERR_SHAPE;
    if (!linear_mfma_supported(SD_DTYPE_BF16, m, n, k, ldy)) return SD_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // scratch: u [n], v [n], row sums [m][2], x = bf16(h gain) [m][k]
    float* u = fold_scratch;
    float* v = u + align_up(n, 64);
    float* stats = v + align_up(n, 64);
    void* xg = stats + 2 * align_up(m, 64);
    if (launch_fold_norm(w, gain, norm_kind == 1 ? beta : nullptr, bias, u, v, n, k, st) != hipSuccess) return SD_ERR_HIP;
    if (launch_norm_prep(h, gain, xg, stats, m, k, st) != hipSuccess) return SD_ERR_HIP;
    NormIn ni;
    ni.kind = norm_kind; ni.stats = stats; ni.parts = 1; ni.u = norm_kind == 1 ? u : nullptr; ni.eps = eps;
    return launch_linear(SD_DTYPE_BF16, xg, w, v, y, m, n, k, ldy, epilogue, ni, NormOut(), ws, st, nullptr) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int32_t sd_linear_resid_norm(const void* x, const void* w, const float* bias, float* y, const float* gain, void* xg,
                             float* stats, int32_t m, int32_t n, int32_t k, void* split_workspace,
                             int64_t split_workspace_bytes, void* hip_stream) {
    if (!x || !w || !y || !gain || !xg || !stats) return SD_ERR_ARG;
    if (split_workspace && ((reinterpret_cast<uintptr_t>(split_workspace) & 255) || split_workspace_bytes <= kSplitTicketBytes))
        return SD_ERR_WORKSPACE;
    const SplitWorkspace ws{split_workspace, split_workspace ? split_workspace_bytes : 0};
    if (m <= 0 || n <= 0 || k <= 0 || !linear_mfma_supported(SD_DTYPE_BF16, m, n, k, n)) return SD_ERR_SHAPE;
    NormOut no;
    no.gain = gain; no.xg = xg; no.stats = stats;
    return launch_linear(SD_DTYPE_BF16, x, w, bias, y, m, n, k, n, EPI_RESID, NormIn(), no, ws, static_cast<hipStream_t>(hip_stream), nullptr) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int32_t sd_set_linear_variant(int32_t variant) {
    linear_mfma_set_variant(variant);
    return SD_OK;
}

int32_t sd_set_linear_split(int32_t split) {
    linear_mfma_set_split(split);
    return SD_OK;
}

int64_t sd_linear_split_ticket_bytes(void) { return kSplitTicketBytes; }

int32_t sd_linear(int32_t dtype, const void* x, const void* w, const float* bias, void* y, int32_t m, int32_t n,
                  int32_t k, int32_t ldy, int32_t epilogue, void* split_workspace, int64_t split_workspace_bytes,
                  void* hip_stream) {
    if (!x || !w || !y) return SD_ERR_ARG;
    if (split_workspace && ((reinterpret_cast<uintptr_t>(split_workspace) & 255) || split_workspace_bytes <= kSplitTicketBytes))
        return SD_ERR_WORKSPACE;
    const SplitWorkspace ws{split_workspace, split_workspace ? split_workspace_bytes : 0};
    if (dtype != SD_DTYPE_F32 && dtype != SD_DTYPE_BF16) return SD_ERR_ARG;
    if (m <= 0 || n <= 0 || k <= 0 || ldy < n || epilogue < 0 || epilogue > 3 || k % 8) return SD_ERR_SHAPE;
    return launch_linear(dtype, x, w, bias, y, m, n, k, ldy, epilogue, NormIn(), NormOut(), ws, static_cast<hipStream_t>(hip_stream), nullptr) == hipSuccess ? SD_OK : SD_ERR_HIP;
}

}  // extern "C"
