// C ABI of libasynclm: sequence state machine, argument checking, memory, launch order.
#include "../../include/asynclm.h"
#include "common.h"
#include "launch.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <new>
#include <vector>

using namespace asynclm;

// Host-side builder of the row table of one pass.
struct PassBuilder {
    ChunkTable t{};
    int G = 1, Hkv = 1, max_keys = 0;
    void clear() { t.rows = t.ngroups = t.ntasks = t.nhead = t.nblocks = 0; max_keys = 0; }
    int tiles_of(int n) const { return (G * n + 31) / 32; }
    // rows, attention tasks, and the attention's partial results (task x kv head x at least 4 key splits) all fit one pass
    bool fits(int n) const {
        return t.rows + n <= CHUNK_MAX && t.ntasks + tiles_of(n) <= CHUNK_MAX_TASKS &&
               (long long)(t.ntasks + tiles_of(n)) * Hkv * 4 <= CHUNK_ATTN_MAX_UNITS;
    }
    // Appends a group of n rows to sequence `seq` (length before: pos0).  forced: see ChunkGroup; `rest` holds the
    // tokens of the rows that are not chosen on the device (n of them if forced == -2, else n - 1).
    void add(int seq, int pos0, int n, int forced, const int32_t* rest, bool want_head) {
        const int row0 = t.rows;
        for (int r = 0; r < n; ++r) {
            ChunkRow& R = t.row[row0 + r];
            R = ChunkRow{};
            R.token = forced == -2 ? rest[r] : (r == 0 ? 0 : rest[r - 1]);
            R.seq = seq; R.pos = pos0 + r; R.row0 = row0; R.n = n;
        }
        ChunkGroup& Gp = t.group[t.ngroups++];
        Gp = ChunkGroup{};
        Gp.seq = seq; Gp.row0 = row0; Gp.n = n; Gp.pos0 = pos0; Gp.forced = forced; Gp.head = want_head ? t.nhead++ : -1;
        for (int tile = 0; tile < tiles_of(n); ++tile) {
            if (tile % 4 == 0) t.block[t.nblocks++] = ChunkTaskBlock{t.ntasks, std::min(4, tiles_of(n) - tile)};
            ChunkTask& T = t.task[t.ntasks++];
            T = ChunkTask{};
            T.seq = seq; T.row0 = row0; T.n = n; T.pos0 = pos0; T.tile = tile;
        }
        t.rows += n;
        max_keys = std::max(max_keys, pos0 + n);
    }
};


struct asynclm_ctx {
    asynclm_config cfg{};
    Geom g{};
    hipStream_t stream = nullptr;
    hipStream_t stream2 = nullptr;      // library-owned: every other kernel of a two-stream decoding step
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    bool pipe_ok = false;               // two workgroups of every single-row kernel fit one compute unit
    unsigned long long* pipe_stamps = nullptr;   // per kernel of the step: see pipe_stamp
    unsigned long long* stamp_done = nullptr;    // [pipe_kernels_max][STAMP_DONE_SLOTS]: see step_stamp_done
    int pipe_kernels = 0;               // kernels of the last step that left time stamps (two streams, or stamp mode); else 0
    int opt_step_stamps = 0;            // stamp mode: one-stream steps run as plain launches and leave time stamps
    bool stamp_now = false;             // the pass being enqueued is such a step
    bool last_step_stamp_mode = false;  // the last step was one
    int pipe_kernels_max = 0;
    unsigned* pipe_go = nullptr;        // [PIPE_REGIONS][PIPE_MAX_WORKGROUPS] hand-over words, one per cache line
    unsigned* pipe_counters = nullptr;  // [pipe_kernels_max] arrival counters, one per cache line
    int device = 0, n_cu = 0;
    bool poisoned = false;
    hipError_t last_hip = hipSuccess;

    const void* embed = nullptr; const float* final_norm = nullptr; const void* lm_head = nullptr;
    std::vector<const float*> attn_norm, ffn_norm;
    std::vector<const void*> wqkv, wo, wgate_up, wdown;

    std::vector<void*> allocs;          // everything from hipMalloc
    void* kv = nullptr;                 // [seq][layer][k|v][Hkv][max_pos][dh] in cfg.dtype
    float* logits = nullptr;            // [max_seqs][V]
    DecodeBuffers b{};
    ChunkBuffers cb{};
    bool chunk_ok = false;              // the matrix-core append path supports this model
    FusedPlan fused{};                  // single-kernel decoding step
    void* layers_dev = nullptr;         // per-layer pointer table of the fused step
    unsigned* bar = nullptr;            // its grid-barrier counters
    unsigned long long* trace = nullptr; // its optional phase time stamps
    bool want_trace = false;
    std::vector<unsigned long long> last_trace;  // raw stamps [stamp][workgroup] of the last profiled fused step
    int last_trace_stamps = 0;
    int32_t* token_host = nullptr;      // pinned, 16 ints: [0..1] staging of read-backs, [4] the token of the running step (early copy)
    hipEvent_t tok_event = nullptr;     // recorded right after the step's token has been chosen
    bool tok_early = false;             // the last decoding step left its token in token_host[4] behind tok_event

    std::vector<int32_t> len;           // host mirror of the sequence lengths
    std::vector<int32_t> nban;          // host mirror of the number of banned token ids per sequence
    std::vector<char> choice_stale;     // the ban list changed after the sequence's greedy token was computed
    PassBuilder pass;                   // row table of the append-chunk pass being built
    int32_t* chosen_host = nullptr;     // pinned, CHUNK_MAX ints
    // pinned staging of what the host uploads on the hot path (a pageable source would make the copy wait for the
    // stream): two copies of the row table and a small ring of ban-list rows, each reused once its event has passed
    ChunkTable* tab_host[2] = {nullptr, nullptr};
    hipEvent_t tab_ev[2] = {nullptr, nullptr};
    int tab_next = 0;
    static constexpr int BAN_RING = 4;
    int32_t* ban_host = nullptr;        // [BAN_RING][1 + BAN_MAX]
    hipEvent_t ban_ev[BAN_RING] = {};
    int ban_next = 0;
    std::vector<char> batch_seen;       // scratch of asynclm_step_batch (sized at create)
    std::vector<int> batch_owner;

    // options
    int opt_chunk = 1, opt_graph = 1, opt_attn_split = 0, opt_chunk_split = 0, opt_fused = 0, opt_attn_mfma_min = 1;
    int opt_pipeline = 0;

    std::map<int, hipGraphExec_t> graphs;   // captured decoding steps by graph_key(), all instantiated by rebuild_graphs()

    // profiling of one step
    bool prof = false;
    std::vector<hipEvent_t> prof_events;
    std::vector<int> prof_class;
};

namespace {

const char* const kClassNames[KC_COUNT] = {
    "begin_step", "embed", "qkv_rope_kvwrite", "attn_decode", "o_proj_residual", "gate_up_swiglu",
    "down_residual", "lm_head", "argmax", "chunk_prep", "chunk_gemm", "chunk_attn", "chunk_misc",
    "fused_step_kernel", "fused:qkv", "fused:qkv_barrier", "fused:attn", "fused:attn_barrier", "fused:merge",
    "fused:merge_barrier", "fused:o_proj", "fused:o_proj_barrier", "fused:gate_up", "fused:gate_up_barrier",
    "fused:down", "fused:down_barrier", "fused:lm_head", "fused:lm_head_barrier"};

// With ASYNCLM_VERBOSE set in the environment, HIP failures are reported on stderr.
void report_hip(const char* where, hipError_t e) {
    if (std::getenv("ASYNCLM_VERBOSE")) std::fprintf(stderr, "[asynclm] %s: %s\n", where, hipGetErrorString(e));
}

int fail_device(asynclm_ctx* c, hipError_t e) {
    report_hip("device call failed", e);
    c->poisoned = true;
    c->last_hip = e;
    return ASYNCLM_E_DEVICE;
}

#define HIPCK(c, expr)                                         \
    do {                                                       \
        hipError_t _e = (expr);                                \
        if (_e != hipSuccess) return fail_device((c), _e);     \
    } while (0)

template <class F>
hipError_t run(asynclm_ctx* c, int kc, F&& f) {
    if (!c->prof) return f();
    hipEvent_t e0, e1;
    hipError_t e;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) return e;
    c->prof_events.push_back(e0); c->prof_events.push_back(e1); c->prof_class.push_back(kc);
    if ((e = hipEventRecord(e0, c->stream)) != hipSuccess) return e;
    if ((e = f()) != hipSuccess) return e;
    return hipEventRecord(e1, c->stream);
}

size_t elem_bytes(const asynclm_ctx* c) { return c->cfg.dtype == ASYNCLM_DTYPE_FP32 ? 4 : 2; }

void* kv_layer_ptr(const asynclm_ctx* c, int layer) {
    return (char*)c->kv + (size_t)layer * c->g.kv_layer_stride * elem_bytes(c);
}

// Attention splits for a context of len_after tokens.  Up to 2048 tokens: at most MERGE_MAX_SPLIT splits, which
// the O projection merges while it stages its input (no merge step at all).  Longer: up to ATTN_MAX_SPLIT
// splits with a merge step of their own.
struct SplitPlan { int nsplit; bool merge_in_oproj; bool mfma; };

SplitPlan pick_nsplit(const asynclm_ctx* c, int len_after, bool single_row_kernel = false) {
    const bool no_v_rows = c->g.kv_v_offset == 0;      // the single-row kernel has nothing to read: matrix cores at any length
    if (!single_row_kernel && c->chunk_ok && (no_v_rows || (c->opt_attn_mfma_min > 0 && len_after >= c->opt_attn_mfma_min))) {
        // attention on the matrix cores: 96 key splits at every length (a wave takes one tile of 32 keys up to 3072 keys,
        // more beyond; waves without keys leave at once), so one captured graph serves every context length.  Measured
        // optima were one tile per wave up to about 96 tiles and 96 splits beyond (more only lengthen the merge).
        int n = 96;
        if (c->opt_attn_split > 0) n = std::max(4, std::min((c->opt_attn_split + 3) / 4 * 4, CHUNK_ATTN_MAX_SPLIT));
        return {n, false, true};
    }
    if (c->opt_attn_split > 0) {
        const int n = c->opt_attn_split < ATTN_MAX_SPLIT ? c->opt_attn_split : ATTN_MAX_SPLIT;
        return {n, n <= 8, false};
    }
    // up to 2048 tokens: a split per 64 positions, at most the 8 that the O projection merges; beyond: a split per
    // 256 positions (one pass of the kernel's inner loop), merged by the last workgroup of each kv head
    const bool merged = len_after <= 2048;
    const int want = merged ? (len_after + 63) / 64 : (len_after + 255) / 256, cap = merged ? 8 : ATTN_MAX_SPLIT;
    int n = 1;
    while (n < want && n < cap) n *= 2;
    return {n, merged, false};
}

// One forward pass of a single row whose token/position are already in the step descriptor.
hipError_t forward_single(asynclm_ctx* c, int seq, bool with_head, SplitPlan sp) {
    const int dt = c->cfg.dtype;
    const Geom& g = c->g;
    hipStream_t s = c->stream;
    hipError_t e;
    if ((e = run(c, KC_EMBED, [&] { return launch_embed(dt, c->embed, c->b, g, s); }))) return e;
    // stamp mode (matrix-core attention plans): every kernel gets six stamp words, six kernels per layer, then the head
    const bool stamps = c->stamp_now && c->pipe_stamps && c->stamp_done;
    int idx = 0;
    PipeSync ps{};
    auto next = [&]() -> const PipeSync* {
        if (!stamps) return nullptr;
        ps.stamps = c->pipe_stamps + (size_t)idx * 6;
        ps.done_wg = c->stamp_done + (size_t)idx * STAMP_DONE_SLOTS;
        ++idx;
        return &ps;
    };
    if (stamps && (e = launch_stamp_init(c->stamp_done, c->pipe_kernels, s))) return e;
    for (int l = 0; l < c->cfg.n_layers; ++l) {
        void* kvl = kv_layer_ptr(c, l);
        const PipeSync* st = next();
        if ((e = run(c, KC_QKV, [&] { return launch_qkv(dt, c->wqkv[l], c->attn_norm[l], kvl, c->b, g, s, st); }))) return e;
        if (sp.mfma) {
            unsigned long long* sw = stamps ? c->pipe_stamps + (size_t)idx * 6 : nullptr;
            unsigned long long* dw = stamps ? c->stamp_done + (size_t)idx * STAMP_DONE_SLOTS : nullptr;
            idx += stamps ? 2 : 0;
            if ((e = run(c, KC_ATTN, [&] { return launch_decode_attn_mfma(c->cb, kvl, sp.nsplit, c->b, g, s, sw, dw); }))) return e;
        } else if ((e = run(c, KC_ATTN, [&] { return launch_attn_decode(dt, kvl, sp.nsplit, sp.merge_in_oproj, c->b, g, s); }))) return e;
        st = next();
        if ((e = run(c, KC_OPROJ, [&] { return launch_oproj(dt, c->wo[l], sp.merge_in_oproj ? sp.nsplit : 0, c->b, g, s, st); }))) return e;
        st = next();
        if ((e = run(c, KC_GATEUP, [&] { return launch_gateup(dt, c->wgate_up[l], c->ffn_norm[l], c->b, g, s, st); }))) return e;
        st = next();
        if ((e = run(c, KC_DOWN, [&] { return launch_down(dt, c->wdown[l], c->b, g, s, st); }))) return e;
    }
    if (with_head) {
        // logits of every sequence live in one array; the kernels pick the row from the descriptor
        const PipeSync* st = next();
        if ((e = run(c, KC_LMHEAD, [&] { return launch_lmhead(dt, c->lm_head, c->final_norm, c->logits, c->b, g, s, st); }))) return e;
        if ((e = run(c, KC_ARGMAX, [&] { return launch_argmax(c->logits, c->b, g, s); }))) return e;
    }
    return hipSuccess;
}

// The same pass with its kernels alternating between two streams, so that two neighbouring kernels run at the same
// time: while kernel n streams its weights and finishes, kernel n + 1 is already resident, has its first weight tiles
// in flight, and waits for kernel n's hand-over counter (PipeSync) before it reads kernel n's output.  Kernel n + 2
// follows kernel n on the same stream, so at most two kernels are in flight; two workgroups of any of them fit one
// compute unit (pipe_ok) and none launches more workgroups than there are compute units, so all workgroups of both
// are resident whatever the order of dispatch and no wait can starve the kernel it waits for.  The attention is the
// single-row kernel with at most 8 key splits, merged by the O projection while it stages its input.
// Visibility without fences (a device-scope release / acquire pair per workgroup writes back and invalidates a whole
// L2 and costs about 10 us once 256 workgroups do it): producers store their results write-through and signal after
// the stores have completed; a consumer reads them with ordinary loads, which cannot hit a stale line, because its
// die's L2 was invalidated when the consumer was dispatched, after every earlier reader of those buffers had ended,
// and nothing reads them again before the producer writes: no vector is updated in place (the residual stream
// alternates between b.x and b.x2), and before its hand-over a kernel reads nothing but weights.
// Measured on the 8B shape (time stamps of asynclm_profile_trace): a hand-over takes about 1 us, but the step is
// slower than the one-stream step (3.7 against 3.4 ms per token): what follows a hand-over - the input vector's round
// trip to memory, the last tiles, the write-through of the results, the counter, the hand-over words - is a chain of
// five to six memory round trips per kernel during which little is streamed, where a kernel of the one-stream step
// overlaps the same chain with its own first 32 MB of weights.  Kept as an option ("pipeline"), off by default.
hipError_t forward_single_pipelined(asynclm_ctx* c, int seq, bool with_head, SplitPlan sp) {
    const int dt = c->cfg.dtype;
    const Geom& g = c->g;
    hipStream_t sa = c->stream, sb = c->stream2;
    hipError_t e;
    if ((e = launch_embed(dt, c->embed, c->b, g, sa))) return e;
    if ((e = hipEventRecord(c->ev_fork, sa))) return e;
    if ((e = hipStreamWaitEvent(sb, c->ev_fork, 0))) return e;
    int idx = 0;
    hipStream_t s = sa;
    PipeSync ps{};
    // kernel k: arrival counter k, signals region k % PIPE_REGIONS, waits on region (k - 1) % PIPE_REGIONS
    auto next = [&]() {
        const size_t region = (size_t)PIPE_MAX_WORKGROUPS * PIPE_LINE_WORDS;
        ps.go_wait = idx > 0 ? c->pipe_go + (size_t)((idx - 1) % PIPE_REGIONS) * region : nullptr;
        ps.go_signal = c->pipe_go + (size_t)(idx % PIPE_REGIONS) * region;
        ps.counter = c->pipe_counters + (size_t)idx * PIPE_LINE_WORDS;
        ps.abort = c->b.pipe_abort;
        ps.error_word = c->b.token_log + 1;
        ps.step = c->b.step;
        ps.wait_kernel = (unsigned)(idx > 0 ? idx - 1 : 0); ps.my_kernel = (unsigned)idx;
        ps.stamps = c->pipe_stamps ? c->pipe_stamps + (size_t)idx * 6 : nullptr;
        s = (idx & 1) ? sb : sa;
        ++idx;
    };
    for (int l = 0; l < c->cfg.n_layers; ++l) {
        void* kvl = kv_layer_ptr(c, l);
        next(); if ((e = launch_qkv(dt, c->wqkv[l], c->attn_norm[l], kvl, c->b, g, s, &ps))) return e;
        next(); if ((e = launch_attn_decode(dt, kvl, sp.nsplit, true, c->b, g, s, &ps))) return e;
        next(); if ((e = launch_oproj(dt, c->wo[l], sp.nsplit, c->b, g, s, &ps, c->b.x2))) return e;
        next(); if ((e = launch_gateup(dt, c->wgate_up[l], c->ffn_norm[l], c->b, g, s, &ps, c->b.x2))) return e;
        next(); if ((e = launch_down(dt, c->wdown[l], c->b, g, s, &ps, c->b.x2))) return e;
    }
    if (with_head) {
        next(); if ((e = launch_lmhead(dt, c->lm_head, c->final_norm, c->logits, c->b, g, s, &ps))) return e;
    }
    if ((e = hipEventRecord(c->ev_join, sb))) return e;
    if ((e = hipStreamWaitEvent(sa, c->ev_join, 0))) return e;
    if (with_head && (e = launch_argmax(c->logits, c->b, g, sa))) return e;
    return hipSuccess;
}

bool use_pipeline(const asynclm_ctx* c, int len_after) {
    // (contexts beyond what 8 key splits of the single-row attention cover take the one-stream step)
    return c->opt_pipeline && c->pipe_ok && !c->prof && c->opt_attn_split == 0 && len_after <= 2048 &&
           5 * c->cfg.n_layers + 1 <= c->pipe_kernels_max && decode_gemv_grid() <= c->n_cu && decode_gemv_grid() <= PIPE_MAX_WORKGROUPS &&
           c->g.Hkv * 8 <= PIPE_MAX_WORKGROUPS;      // at most 8 key splits reach this step
}

// Captured steps.  The kernels read token, position and sequence from the step descriptor, so a graph depends only on
// the launch geometry: the attention plan, whether the pass ends with the output head, one or two streams.
int graph_key(SplitPlan sp, bool with_head, bool pipelined) {
    return ((((sp.nsplit << 1 | (sp.merge_in_oproj ? 1 : 0)) << 1 | (sp.mfma ? 1 : 0)) << 1 | (with_head ? 1 : 0)) << 1) | (pipelined ? 1 : 0);
}

hipError_t capture_step(asynclm_ctx* c, SplitPlan sp, bool with_head, bool pipelined, hipGraphExec_t* out) {
    hipError_t e;
    hipGraph_t graph = nullptr;
    if ((e = hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed))) return e;
    if (pipelined) e = forward_single_pipelined(c, 0, with_head, sp);
    else {
        // stamp mode: the captured kernels carry their stamp words (the graphs are rebuilt when the option changes)
        c->stamp_now = c->opt_step_stamps && sp.mfma;
        if (c->stamp_now) c->pipe_kernels = 6 * c->cfg.n_layers + (with_head ? 1 : 0);
        e = forward_single(c, 0, with_head, sp);
        c->stamp_now = false;
    }
    hipError_t e2 = hipStreamEndCapture(c->stream, &graph);
    if (e) { if (graph) hipGraphDestroy(graph); return e; }
    if (e2) return e2;
    e = hipGraphInstantiate(out, graph, nullptr, nullptr, 0);
    hipGraphDestroy(graph);
    return e;
}

// Instantiates every graph that a decoding step can need under the current options (all attention plans that occur
// up to max_positions), so that no decoding step captures, instantiates or allocates.  Called by asynclm_create and by
// the options that change the launch geometry.
hipError_t rebuild_graphs(asynclm_ctx* c) {
    for (auto& kv : c->graphs) hipGraphExecDestroy(kv.second);
    c->graphs.clear();
    if (!c->opt_graph || !c->stream || c->opt_fused) return hipSuccess;
    const bool was_prof = c->prof;
    c->prof = false;
    hipError_t e = hipSuccess;
    for (int len_after = 1; len_after <= c->cfg.max_positions && !e; ++len_after) {
        const bool pipelined = use_pipeline(c, len_after);
        const SplitPlan sp = pick_nsplit(c, len_after, pipelined);
        for (int with_head = 0; with_head < 2 && !e; ++with_head) {
            const int key = graph_key(sp, with_head != 0, pipelined);
            if (c->graphs.count(key)) continue;
            hipGraphExec_t exec = nullptr;
            if ((e = capture_step(c, sp, with_head != 0, pipelined, &exec)) == hipSuccess) c->graphs.emplace(key, exec);
        }
    }
    c->prof = was_prof;
    return e;
}

// The greedy token of a sequence is computed when a forward pass ends; if the ban list changed since, it is
// recomputed from the (unchanged) logits before it is used.
hipError_t refresh_choice(asynclm_ctx* c, int seq) {
    if (!c->choice_stale[seq]) return hipSuccess;
    c->choice_stale[seq] = 0;
    return launch_argmax(c->logits, c->b, c->g, c->stream, seq);
}

hipError_t step_one_token(asynclm_ctx* c, int seq, int forced, bool with_head) {
    hipError_t e;
    c->tok_early = false;
    if (forced < 0 && (e = refresh_choice(c, seq))) return e;
    if (c->opt_fused && c->nban[seq] == 0) {      // the single-kernel step has no token mask
        FusedLaunch L{};
        L.layers_dev = c->layers_dev; L.n_layers = c->cfg.n_layers;
        L.embed = c->embed; L.final_norm = c->final_norm; L.lm_head = c->lm_head;
        L.seq = seq; L.forced = forced; L.with_head = with_head;
        {
            SplitPlan sp = pick_nsplit(c, c->len[seq] + 1);
            if (!sp.merge_in_oproj) sp.nsplit = c->fused.nsplit;          // long context: every workgroup takes a split
            if (sp.nsplit > c->fused.nsplit) sp.nsplit = c->fused.nsplit;
            L.nsplit = sp.nsplit; L.merge_in_stage = sp.merge_in_oproj;
        }
        L.logits = c->logits + (size_t)seq * c->g.V; L.bar = c->bar; L.trace = c->want_trace ? c->trace : nullptr;
        if ((e = launch_decode_fused(c->cfg.dtype, c->fused, L, c->b, c->g, c->stream))) return e;
        c->len[seq] += 1;
        return hipSuccess;
    }
    const bool pipelined = use_pipeline(c, c->len[seq] + 1);
    const SplitPlan sp = pick_nsplit(c, c->len[seq] + 1, pipelined);
    // the chosen token also goes to pinned host memory, and an event marks the point: asynclm_decode_step waits for that
    // event only, so the host has the token while the forward pass is still running
    if ((e = run(c, KC_BEGIN, [&] { return launch_begin_step(c->b, seq, forced, c->tok_event ? c->token_host + 4 : nullptr, c->stream); }))) return e;
    if (c->tok_event && !c->prof) {
        if ((e = hipEventRecord(c->tok_event, c->stream))) return e;
        c->tok_early = true;
    }
    c->pipe_kernels = pipelined ? 5 * c->cfg.n_layers + (with_head ? 1 : 0) : 0;
    const bool stamp_mode = c->opt_step_stamps && !pipelined && sp.mfma && !c->prof;
    if (stamp_mode) c->pipe_kernels = 6 * c->cfg.n_layers + (with_head ? 1 : 0);
    c->last_step_stamp_mode = stamp_mode;
    auto g_it = (c->opt_graph && !c->prof) ? c->graphs.find(graph_key(sp, with_head, pipelined)) : c->graphs.end();
    if (g_it != c->graphs.end()) e = hipGraphLaunch(g_it->second, c->stream);
    else if (pipelined) e = forward_single_pipelined(c, seq, with_head, sp);
    else {
        c->stamp_now = stamp_mode;
        e = forward_single(c, seq, with_head, sp);
        c->stamp_now = false;
    }
    if (e) return e;
    c->len[seq] += 1;
    return hipSuccess;
}

template <class T>
hipError_t dev_alloc(asynclm_ctx* c, T** p, size_t count) {
    void* v = nullptr;
    hipError_t e = hipMalloc(&v, count * sizeof(T) > 0 ? count * sizeof(T) : 16);
    if (e != hipSuccess) return e;
    c->allocs.push_back(v);
    *p = (T*)v;
    return hipSuccess;
}

bool config_ok(const asynclm_config* k) {
    if (k->n_layers <= 0 || k->d_model <= 0 || k->n_q_heads <= 0 || k->n_kv_heads <= 0 || k->ffn <= 0 || k->vocab <= 0) return false;
    if (k->head_dim != 64 && k->head_dim != 128) return false;
    if (k->n_q_heads % k->n_kv_heads) return false;
    const int grp = k->n_q_heads / k->n_kv_heads;
    if (grp != 1 && grp != 2 && grp != 4 && grp != 8) return false;
    if (k->d_model % 8 || k->ffn % 8) return false;
    if (k->dtype != ASYNCLM_DTYPE_FP32 && k->dtype != ASYNCLM_DTYPE_BF16) return false;
    if (k->max_seqs < 1 || k->max_positions < 1) return false;
    if (k->kv_format != ASYNCLM_KV_AUTO &&
        !((k->kv_format == ASYNCLM_KV_BF16 || k->kv_format == ASYNCLM_KV_PAIR_ROWS) && k->dtype == ASYNCLM_DTYPE_BF16)) return false;
    if (!(k->rms_eps >= 0.f) || !(k->rope_theta > 0.f)) return false;
    return true;
}

int check_seq(const asynclm_ctx* c, int32_t seq) {
    if (!c) return ASYNCLM_E_INVAL;
    if (c->poisoned) return ASYNCLM_E_DEVICE;
    if (seq < 0 || seq >= c->cfg.max_seqs) return ASYNCLM_E_INVAL;
    return ASYNCLM_OK;
}

int check_tokens(const asynclm_ctx* c, const int32_t* t, int32_t n) {
    if (!t || n <= 0) return ASYNCLM_E_INVAL;
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= c->cfg.vocab) return ASYNCLM_E_INVAL;
    return ASYNCLM_OK;
}

// Split-K factors of the four products of a layer (workgroups = N/32 * S, each of 4 waves).
struct ChunkSplits { int qkv, o, gu, down; };

// A product with N output rows and K columns over MT row tiles runs (N/128) * (row blocks) * S workgroups, one per
// compute unit at a time: S = the split that comes closest to one workgroup per unit, with at least two
// 128-column blocks per workgroup, within the capacity of the partial planes.
int pick_gemm_split(const asynclm_ctx* c, int N, int K, int MT) {
    const int row_blocks = MT <= 4 ? 1 : (MT + 7) / 8;          // as launch_chunk_gemm tiles the rows
    const int tiles = N / 128 * row_blocks, nblk = K / 128;
    const int smax = std::min(CHUNK_GEMM_MAX_SPLIT, std::max(1, nblk / 2));
    int s;
    if (MT <= 3) {
        s = std::max(1, std::min((c->n_cu + tiles / 2) / tiles, smax));
    } else {
        // wide passes are bound by the matrix cores: the workgroups run in rounds of one per compute unit, each taking
        // its k-blocks plus about one and a half blocks' time of prologue and epilogue; every split also costs a
        // partial plane to write and read back
        // (a plane of 512 x 4096 floats, written and read back, costs about as much as one k-block of a workgroup)
        s = 1;
        double best = 0;
        const double plane = 0.9 * ((double)MT * 32 * N) / (512.0 * 4096.0);
        for (int k = 1; k <= smax; ++k) {
            const int rounds = (tiles * k + c->n_cu - 1) / c->n_cu;
            const double cost = rounds * ((double)nblk / k + 1.5) + plane * (k - 1);
            if (k == 1 || cost < best) { best = cost; s = k; }
        }
    }
    if (c->opt_chunk_split > 0) s = std::min(c->opt_chunk_split, std::max(1, nblk));
    while (s > 1 && (size_t)s * MT * 32 * N > c->cb.part_capacity) --s;
    return s;
}

ChunkSplits chunk_splits(const asynclm_ctx* c, int MT) {
    const Geom& g = c->g;
    // the gate/up product of a wide pass is never split (unless forced): split-K would lose its SwiGLU epilogue
    const int gu = MT > 3 && c->opt_chunk_split == 0 ? 1 : pick_gemm_split(c, 2 * g.F, g.d, MT);
    return {pick_gemm_split(c, (g.Hq + 2 * g.Hkv) * g.dh, g.d, MT), pick_gemm_split(c, g.d, g.Hq * g.dh, MT), gu,
            pick_gemm_split(c, g.d, g.F, MT)};
}

// Key splits of the chunk attention: about two 32-key tiles per wave, a multiple of 4, no more than fill the
// device eight waves deep (a large pass has enough tasks: more splits only add partial results to write and
// merge), within the capacity of the partial-result buffers.
int pick_chunk_attn_split(const asynclm_ctx* c, int max_keys, int ntasks) {
    const int tiles = (max_keys + 31) / 32;
    int n = ((tiles + 1) / 2 + 3) / 4 * 4;
    n = std::max(4, std::min(n, CHUNK_ATTN_MAX_SPLIT));
    const long long groups = (long long)ntasks * c->g.Hkv;
    const int fill = (int)std::max(4LL, 8LL * c->n_cu / groups / 4 * 4);
    n = std::min(n, fill);
    while (n > 4 && groups * n > CHUNK_ATTN_MAX_UNITS) n -= 4;
    return n;
}

// One forward pass over the rows of `pb` (1..CHUNK_MAX rows in any number of groups).  Groups that want logits
// get them from the single-row head kernels (one group) or from one more product on the matrix cores (several).
hipError_t forward_chunk(asynclm_ctx* c, const PassBuilder& pb) {
    const Geom& g = c->g;
    const ChunkBuffers& cb = c->cb;
    hipStream_t s = c->stream;
    const ChunkTable& t = pb.t;
    const int rows = t.rows, MT = (rows + 31) / 32;
    const ChunkSplits sp = chunk_splits(c, MT);
    const int nqkv = (g.Hq + 2 * g.Hkv) * g.dh, qd = g.Hq * g.dh;
    const int asplit = pick_chunk_attn_split(c, pb.max_keys, t.ntasks);
    // passes made of large groups (at least 16 tasks, three or more per block on average) share keys and values
    // between the tasks of a block; their key splits: about two workgroups per compute unit, at least four tiles each
    const bool wide_attn = t.ntasks >= 16 && t.ntasks >= 3 * t.nblocks;
    int wsplit = 1;
    if (wide_attn) {
        const long long wgs = (long long)t.nblocks * g.Hkv;
        wsplit = (int)std::max(1LL, std::min<long long>((2LL * c->n_cu + wgs - 1) / wgs, ((pb.max_keys + 31) / 32 + 3) / 4));
        wsplit = std::min(wsplit, CHUNK_ATTN_MAX_SPLIT);
        while (wsplit > 1 && (long long)t.ntasks * g.Hkv * wsplit > CHUNK_ATTN_MAX_UNITS) --wsplit;
    }
    const int dt = c->cfg.dtype;
    hipError_t e;
    {   // through pinned memory: the copy is asynchronous and the host goes on enqueuing the pass
        const int i = c->tab_next;
        const size_t bytes = offsetof(ChunkTable, row) + sizeof(ChunkRow) * rows;
        if ((e = hipEventSynchronize(c->tab_ev[i]))) return e;         // the upload that last used this copy has finished
        std::memcpy(c->tab_host[i], &t, bytes);
        if ((e = hipMemcpyAsync(cb.tab, c->tab_host[i], bytes, hipMemcpyHostToDevice, s))) return e;
        if ((e = hipEventRecord(c->tab_ev[i], s))) return e;
        c->tab_next = i ^ 1;
    }
    if ((e = run(c, KC_BEGIN, [&] { return launch_begin_chunk(cb, c->b, t.ngroups, s); }))) return e;
    if ((e = run(c, KC_CHUNK_PREP, [&] { return launch_chunk_embed(c->embed, cb, rows, g, s); }))) return e;
    for (int l = 0; l < c->cfg.n_layers; ++l) {
        void* kvl = kv_layer_ptr(c, l);
        if ((e = run(c, KC_CHUNK_PREP, [&] { return launch_chunk_resid_norm(cb, l > 0, sp.down, MT, c->attn_norm[l], rows, g, s); }))) return e;
        if ((e = run(c, KC_CHUNK_GEMM, [&] { return launch_chunk_gemm(c->wqkv[l], nqkv, g.d, cb.nrm_hi, cb.nrm_lo, cb, sp.qkv, MT, s); }))) return e;
        if ((e = run(c, KC_CHUNK_PREP, [&] { return launch_chunk_rope_kv(cb, sp.qkv, kvl, c->b, rows, MT, g, s); }))) return e;
        if (wide_attn) { if ((e = run(c, KC_CHUNK_ATTN, [&] { return launch_chunk_attn_wide(cb, kvl, wsplit, t.ntasks, t.nblocks, g, s); }))) return e; }
        else if ((e = run(c, KC_CHUNK_ATTN, [&] { return launch_chunk_attn(cb, kvl, asplit, t.ntasks, g, s); }))) return e;
        if ((e = run(c, KC_CHUNK_GEMM, [&] { return launch_chunk_gemm(c->wo[l], g.d, qd, cb.att_hi, cb.att_lo, cb, sp.o, MT, s); }))) return e;
        if ((e = run(c, KC_CHUNK_PREP, [&] { return launch_chunk_resid_norm(cb, true, sp.o, MT, c->ffn_norm[l], rows, g, s); }))) return e;
        if (sp.gu == 1) {                 // no split-K: the SwiGLU is the product's epilogue
            if ((e = run(c, KC_CHUNK_GEMM, [&] { return launch_chunk_gemm_swiglu(c->wgate_up[l], g.F, g.d, cb.nrm_hi, cb.nrm_lo, cb, MT, s); }))) return e;
        } else {
            if ((e = run(c, KC_CHUNK_GEMM, [&] { return launch_chunk_gemm(c->wgate_up[l], 2 * g.F, g.d, cb.nrm_hi, cb.nrm_lo, cb, sp.gu, MT, s); }))) return e;
            if ((e = run(c, KC_CHUNK_PREP, [&] { return launch_chunk_swiglu(cb, sp.gu, MT, rows, g, s); }))) return e;
        }
        if ((e = run(c, KC_CHUNK_GEMM, [&] { return launch_chunk_gemm(c->wdown[l], g.d, g.F, cb.act_hi, cb.act_lo, cb, sp.down, MT, s); }))) return e;
    }
    const bool head_on_mfma = t.nhead > 1 && g.V % 128 == 0 && (size_t)((t.nhead + 31) / 32) * 32 * g.V <= cb.part_capacity;
    if (head_on_mfma) {
        const int MTh = (t.nhead + 31) / 32;
        if ((e = run(c, KC_CHUNK_MISC, [&] { return launch_chunk_head_rows(cb, sp.down, MT, c->final_norm, t.ngroups, g, s); }))) return e;
        if ((e = run(c, KC_LMHEAD, [&] { return launch_chunk_gemm(c->lm_head, g.V, g.d, cb.nrm_hi, cb.nrm_lo, cb, 1, MTh, s); }))) return e;
        if ((e = run(c, KC_ARGMAX, [&] { return launch_chunk_logits(cb, MTh, c->logits, c->b, t.ngroups, g, s); }))) return e;
    } else {
        for (int gi = 0; gi < t.ngroups; ++gi) {
            if (t.group[gi].head < 0) continue;
            const int seq = t.group[gi].seq;
            if ((e = run(c, KC_CHUNK_MISC, [&] { return launch_chunk_last_row(cb, sp.down, MT, gi, c->b, g, s); }))) return e;
            if ((e = run(c, KC_LMHEAD, [&] { return launch_lmhead(dt, c->lm_head, c->final_norm, c->logits, c->b, g, s); }))) return e;
            if ((e = run(c, KC_ARGMAX, [&] { return launch_argmax(c->logits, c->b, g, s); }))) return e;
        }
    }
    for (int gi = 0; gi < t.ngroups; ++gi) c->len[t.group[gi].seq] = t.group[gi].pos0 + t.group[gi].n;
    return hipSuccess;
}

// Append n >= 1 tokens to a sequence and leave logits for the token after them.
int append_tokens(asynclm_ctx* c, int seq, const int32_t* tokens, int n) {
    const int chunk = c->chunk_ok ? std::min(c->opt_chunk, CHUNK_MAX) : 1;
    int i = 0;
    while (i < n) {
        const int rows = std::min(chunk, n - i);
        const bool last = i + rows == n;
        if (rows == 1) {
            HIPCK(c, step_one_token(c, seq, tokens[i], last));
        } else {
            PassBuilder& pb = c->pass;
            pb.clear();
            pb.add(seq, c->len[seq], rows, -2, tokens + i, last);
            HIPCK(c, forward_chunk(c, pb));
        }
        i += rows;
    }
    return ASYNCLM_OK;
}

}  // namespace

extern "C" {

int asynclm_create(asynclm_ctx** out, const asynclm_config* cfg, const asynclm_weights* w, void* hip_stream) {
    if (out) *out = nullptr;
    if (!out || !cfg || !w) return ASYNCLM_E_INVAL;
    if (!config_ok(cfg)) return ASYNCLM_E_INVAL;
    if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
        !w->wgate_up || !w->wdown)
        return ASYNCLM_E_INVAL;
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->wgate_up[l] || !w->wdown[l])
            return ASYNCLM_E_INVAL;

    asynclm_ctx* c = new (std::nothrow) asynclm_ctx();
    if (!c) return ASYNCLM_E_NOMEM;
    hipError_t e0;
    c->cfg = *cfg;
    c->stream = (hipStream_t)hip_stream;
    if (!c->stream) c->opt_graph = 0;   // the null stream cannot be captured
    if ((e0 = hipGetDevice(&c->device)) != hipSuccess) { report_hip("hipGetDevice", e0); delete c; return ASYNCLM_E_DEVICE; }
    if ((e0 = hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device)) != hipSuccess || c->n_cu < 1) {
        report_hip("hipDeviceGetAttribute", e0); delete c; return ASYNCLM_E_DEVICE;
    }

    c->embed = w->embed; c->final_norm = w->final_norm; c->lm_head = w->lm_head;
    for (int l = 0; l < cfg->n_layers; ++l) {
        c->attn_norm.push_back(w->attn_norm[l]); c->ffn_norm.push_back(w->ffn_norm[l]);
        c->wqkv.push_back(w->wqkv[l]); c->wo.push_back(w->wo[l]);
        c->wgate_up.push_back(w->wgate_up[l]); c->wdown.push_back(w->wdown[l]);
    }

    Geom& g = c->g;
    g.d = cfg->d_model; g.Hq = cfg->n_q_heads; g.Hkv = cfg->n_kv_heads; g.dh = cfg->head_dim;
    g.F = cfg->ffn; g.V = cfg->vocab; g.max_pos = (cfg->max_positions + 31) / 32 * 32; g.eps = cfg->rms_eps;
    g.scale = (float)(1.0 / std::sqrt((double)cfg->head_dim));
    {
        const bool pair = cfg->dtype == ASYNCLM_DTYPE_BF16 && cfg->kv_format != ASYNCLM_KV_BF16;
        // the matrix-core append path: bf16 weights, paired cache, head_dim 128, 128-aligned inner sizes
        c->chunk_ok = pair && g.dh == 128 && g.d % 128 == 0 && g.F % 128 == 0 && g.d <= 8192;
        const size_t plane = (size_t)g.max_pos * g.dh * g.Hkv;
        g.kv_head_stride = (size_t)g.max_pos * g.dh;
        // row-major values: every model but those of the append path, whose attention (decoding steps included) reads
        // the transposed planes only; PAIR_ROWS keeps both
        const bool v_rows = !c->chunk_ok || cfg->kv_format == ASYNCLM_KV_PAIR_ROWS;
        g.kv_lo_offset = pair ? plane : 0;
        g.kv_v_offset = v_rows ? (pair ? 2 * plane : plane) : 0;
        const size_t row_planes = (pair ? 2 : 1) * (v_rows ? 2 : 1);
        g.kv_vt_offset = c->chunk_ok ? row_planes * plane : 0;
        g.kv_layer_stride = (row_planes + (c->chunk_ok ? 2 : 0)) * plane;
        g.kv_seq_stride = g.kv_layer_stride * cfg->n_layers;
        if (c->chunk_ok) c->opt_chunk = CHUNK_MAX;
    }
    c->len.assign(cfg->max_seqs, 0);
    c->nban.assign(cfg->max_seqs, 0);
    c->choice_stale.assign(cfg->max_seqs, 0);

    auto bail = [&](int code) { asynclm_destroy(c); return code; };
    hipError_t e;
#define ALLOC(ptr, count) if ((e = dev_alloc(c, &(ptr), (count))) != hipSuccess) { report_hip("hipMalloc " #ptr, e); return bail(e == hipErrorOutOfMemory ? ASYNCLM_E_NOMEM : ASYNCLM_E_DEVICE); }
    {
        char* kvp = nullptr;
        ALLOC(kvp, g.kv_seq_stride * (size_t)cfg->max_seqs * elem_bytes(c));
        c->kv = kvp;
    }
    ALLOC(c->logits, (size_t)cfg->max_seqs * g.V);
    ALLOC(c->b.step, 1);
    ALLOC(c->b.seq_state, (size_t)cfg->max_seqs);
    ALLOC(c->b.token_log, 2);        // [0] chosen token, [1] set when a fused step gave up at a grid barrier
    ALLOC(c->b.x, (size_t)g.d);
    ALLOC(c->b.x2, (size_t)g.d);
    ALLOC(c->b.q, (size_t)g.Hq * g.dh);
    ALLOC(c->b.o, (size_t)g.Hq * g.dh);
    ALLOC(c->b.a, (size_t)g.F);
    ALLOC(c->b.part_acc, (size_t)g.Hq * ATTN_MAX_SPLIT * g.dh);
    ALLOC(c->b.part_ml, (size_t)g.Hq * ATTN_MAX_SPLIT * 2);
    ALLOC(c->b.attn_counters, (size_t)g.Hkv);
    ALLOC(c->b.amax_v, (size_t)ARGMAX_MAX_BLOCKS);
    ALLOC(c->b.amax_i, (size_t)ARGMAX_MAX_BLOCKS);
    ALLOC(c->b.amax_counter, 1);
    ALLOC(c->b.banned, (size_t)cfg->max_seqs * (1 + BAN_MAX));
    c->pipe_kernels_max = 6 * cfg->n_layers + 2;      // two-stream step: 5 per layer; stamp mode of the one-stream step: 6
    ALLOC(c->b.pipe_abort, (size_t)PIPE_LINE_WORDS);
    ALLOC(c->pipe_go, (size_t)PIPE_REGIONS * PIPE_MAX_WORKGROUPS * PIPE_LINE_WORDS);
    ALLOC(c->pipe_counters, (size_t)c->pipe_kernels_max * PIPE_LINE_WORDS);
    ALLOC(c->pipe_stamps, (size_t)c->pipe_kernels_max * 6);
    ALLOC(c->stamp_done, (size_t)c->pipe_kernels_max * STAMP_DONE_SLOTS);
    if (c->chunk_ok) {
        ChunkBuffers& cb = c->cb;
        const size_t M = CHUNK_MAX, qd = (size_t)g.Hq * g.dh;
        // split-K partial planes: every split of the widest product for passes of up to 96 rows (bound by the weight
        // stream: many splits), two for the largest pass (bound by the matrix cores: few), the output head for one
        // row per group
        const size_t wmax = std::max(std::max((size_t)2 * g.F, (size_t)(g.Hq + 2 * g.Hkv) * g.dh), (size_t)g.d);
        cb.part_capacity = std::max(std::max((size_t)96 * CHUNK_GEMM_MAX_SPLIT * wmax, 2 * M * wmax), (size_t)CHUNK_MAX_TASKS * g.V);
        if ((e = chunk_init()) != hipSuccess) { report_hip("chunk_init", e); return bail(ASYNCLM_E_DEVICE); }
        cb.q_cols = (g.Hq / g.Hkv) * CHUNK_MAX + 32;
        const size_t qn = (size_t)g.Hkv * cb.q_cols * g.dh;
        c->pass.G = g.Hq / g.Hkv; c->pass.Hkv = g.Hkv;
        ALLOC(cb.tab, 1);
        ALLOC(cb.chosen, M);
        ALLOC(cb.x, M * g.d);
        ALLOC(cb.nrm_hi, M * g.d); ALLOC(cb.nrm_lo, M * g.d);
        ALLOC(cb.att_hi, M * qd); ALLOC(cb.att_lo, M * qd);
        ALLOC(cb.act_hi, M * g.F); ALLOC(cb.act_lo, M * g.F);
        ALLOC(cb.q_hi, qn); ALLOC(cb.q_lo, qn);
        ALLOC(cb.part, cb.part_capacity);
        ALLOC(cb.attn_o, (size_t)CHUNK_ATTN_MAX_UNITS * g.dh * 32);
        ALLOC(cb.attn_ml, (size_t)CHUNK_ATTN_MAX_UNITS * 64);
        // rows beyond the current chunk are multiplied into discarded columns only, but must stay finite
        if (hipMemset(cb.tab, 0, sizeof(ChunkTable)) || hipMemset(cb.chosen, 0, M * 4) || hipMemset(cb.x, 0, M * g.d * 4) || hipMemset(cb.nrm_hi, 0, M * g.d * 2) ||
            hipMemset(cb.nrm_lo, 0, M * g.d * 2) || hipMemset(cb.att_hi, 0, M * qd * 2) || hipMemset(cb.att_lo, 0, M * qd * 2) ||
            hipMemset(cb.act_hi, 0, M * g.F * 2) || hipMemset(cb.act_lo, 0, M * g.F * 2) || hipMemset(cb.q_hi, 0, qn * 2) ||
            hipMemset(cb.q_lo, 0, qn * 2))
            return bail(ASYNCLM_E_DEVICE);
    }
    // cache rows that were never written are read (and masked) by the chunk attention: keep them finite
    if (hipMemset(c->kv, 0, g.kv_seq_stride * (size_t)cfg->max_seqs * elem_bytes(c)) != hipSuccess) return bail(ASYNCLM_E_DEVICE);
    float *rc = nullptr, *rs = nullptr;
    const size_t half = g.dh / 2, rope_n = (size_t)g.max_pos * half;
    ALLOC(rc, rope_n);
    ALLOC(rs, rope_n);
#undef ALLOC
    c->b.rope_cos = rc; c->b.rope_sin = rs;

    // rotary table: angle(pos, i) = pos * theta^(-2i/dh), formed in double, stored as fp32
    {
        std::vector<float> hc(rope_n), hs(rope_n);
        std::vector<double> inv(half);
        for (size_t i = 0; i < half; ++i) inv[i] = std::pow((double)cfg->rope_theta, -2.0 * (double)i / (double)g.dh);
        for (int p = 0; p < g.max_pos; ++p)
            for (size_t i = 0; i < half; ++i) {
                const double ang = (double)p * inv[i];
                hc[(size_t)p * half + i] = (float)std::cos(ang);
                hs[(size_t)p * half + i] = (float)std::sin(ang);
            }
        if (hipMemcpy(rc, hc.data(), rope_n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(rs, hs.data(), rope_n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
            return bail(ASYNCLM_E_DEVICE);
    }
    if (hipMemset(c->b.seq_state, 0, sizeof(SeqState) * cfg->max_seqs) != hipSuccess ||
        hipMemset(c->b.attn_counters, 0, sizeof(int32_t) * g.Hkv) != hipSuccess ||
        hipMemset(c->b.amax_counter, 0, sizeof(int32_t)) != hipSuccess ||
        hipMemset(c->b.banned, 0, sizeof(int32_t) * cfg->max_seqs * (1 + BAN_MAX)) != hipSuccess ||
        hipMemset(c->b.step, 0, sizeof(StepDesc)) != hipSuccess || hipMemset(c->b.token_log, 0, 2 * sizeof(int32_t)) != hipSuccess)
        return bail(ASYNCLM_E_DEVICE);
    if (hipHostMalloc((void**)&c->token_host, 64, hipHostMallocDefault) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
    std::memset(c->token_host, 0, 64);
    if (hipEventCreateWithFlags(&c->tok_event, hipEventDisableTiming) != hipSuccess) return bail(ASYNCLM_E_DEVICE);
    if (hipMemset(c->b.pipe_abort, 0, sizeof(unsigned) * PIPE_LINE_WORDS) != hipSuccess ||
        hipMemset(c->pipe_go, 0xff, sizeof(unsigned) * PIPE_REGIONS * PIPE_MAX_WORKGROUPS * PIPE_LINE_WORDS) != hipSuccess ||
        hipMemset(c->pipe_counters, 0, sizeof(unsigned) * c->pipe_kernels_max * PIPE_LINE_WORDS) != hipSuccess)
        return bail(ASYNCLM_E_DEVICE);
    if (c->stream) {     // second stream of the two-stream decoding step (default priority, as every stream here)
        if (hipStreamCreateWithFlags(&c->stream2, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess)
            return bail(ASYNCLM_E_DEVICE);
    }
    if (hipHostMalloc((void**)&c->chosen_host, sizeof(int32_t) * CHUNK_MAX, hipHostMallocDefault) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
    for (int i = 0; i < 2; ++i)
        if (hipHostMalloc((void**)&c->tab_host[i], sizeof(ChunkTable), hipHostMallocDefault) != hipSuccess ||
            hipEventCreateWithFlags(&c->tab_ev[i], hipEventDisableTiming) != hipSuccess)
            return bail(ASYNCLM_E_NOMEM);
    if (hipHostMalloc((void**)&c->ban_host, sizeof(int32_t) * asynclm_ctx::BAN_RING * (1 + BAN_MAX), hipHostMallocDefault) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
    for (int i = 0; i < asynclm_ctx::BAN_RING; ++i)
        if (hipEventCreateWithFlags(&c->ban_ev[i], hipEventDisableTiming) != hipSuccess) return bail(ASYNCLM_E_DEVICE);
    c->batch_seen.assign(cfg->max_seqs, 0);
    c->batch_owner.reserve(CHUNK_MAX_TASKS + 1);
    // fused decoding step: pointer table, barrier counters, launch plan
    {
        std::vector<const void*> tab;
        for (int l = 0; l < cfg->n_layers; ++l) {
            tab.push_back(c->attn_norm[l]); tab.push_back(c->wqkv[l]); tab.push_back(c->wo[l]);
            tab.push_back(c->ffn_norm[l]); tab.push_back(c->wgate_up[l]); tab.push_back(c->wdown[l]);
            tab.push_back(kv_layer_ptr(c, l));
        }
        char* tabd = nullptr;
        if ((e = dev_alloc(c, &tabd, tab.size() * sizeof(void*))) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
        c->layers_dev = tabd;
        if ((e = dev_alloc(c, &c->bar, (size_t)FUSED_BAR_WORDS)) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
        
        if (hipMemcpy(tabd, tab.data(), tab.size() * sizeof(void*), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemset(c->bar, 0, FUSED_BAR_WORDS * sizeof(unsigned)) != hipSuccess)
            return bail(ASYNCLM_E_DEVICE);
        if ((e = fused_init(cfg->dtype, g, &c->fused)) != hipSuccess) { report_hip("fused_init", e); return bail(ASYNCLM_E_DEVICE); }
        if (g.kv_v_offset == 0) c->fused.supported = false;     // its attention reads the values row by row
        c->opt_fused = 0;      // opt-in (set_option "fused"): the per-operation kernels are currently faster
        if (c->fused.supported && (e = dev_alloc(c, &c->trace, (size_t)FUSED_TRACE_MAX * c->fused.grid)) != hipSuccess) return bail(ASYNCLM_E_NOMEM);
    }
    const int max_k = g.F > g.d ? (g.F > g.Hq * g.dh ? g.F : g.Hq * g.dh) : (g.d > g.Hq * g.dh ? g.d : g.Hq * g.dh);
    if ((e = decode_init(cfg->dtype, max_k)) != hipSuccess) { report_hip("decode_init", e); return bail(ASYNCLM_E_DEVICE); }
    c->pipe_ok = c->stream2 && g.kv_v_offset != 0 && decode_pipeline_fits(cfg->dtype, g, g.kv_lo_offset != 0);
    if (const char* pv = std::getenv("ASYNCLM_PIPELINE")) c->opt_pipeline = (std::atoi(pv) != 0 && c->pipe_ok) ? 1 : 0;
    if (std::getenv("ASYNCLM_VERBOSE")) std::fprintf(stderr, "[asynclm] two-stream step: fits %d, on %d\n", (int)c->pipe_ok, c->opt_pipeline);
    if ((e = rebuild_graphs(c)) != hipSuccess) { report_hip("capture of the decoding steps", e); return bail(ASYNCLM_E_DEVICE); }
    if ((e = hipDeviceSynchronize()) != hipSuccess) { report_hip("hipDeviceSynchronize", e); return bail(ASYNCLM_E_DEVICE); }
    *out = c;
    return ASYNCLM_OK;
}

int asynclm_destroy(asynclm_ctx* c) {
    if (!c) return ASYNCLM_OK;
    hipStreamSynchronize(c->stream);
    for (auto& kv : c->graphs) hipGraphExecDestroy(kv.second);
    for (hipEvent_t ev : c->prof_events) hipEventDestroy(ev);
    for (void* p : c->allocs) hipFree(p);
    if (c->token_host) hipHostFree(c->token_host);
    if (c->tok_event) hipEventDestroy(c->tok_event);
    if (c->stream2) { hipStreamSynchronize(c->stream2); hipStreamDestroy(c->stream2); }
    if (c->ev_fork) hipEventDestroy(c->ev_fork);
    if (c->ev_join) hipEventDestroy(c->ev_join);
    if (c->chosen_host) hipHostFree(c->chosen_host);
    for (int i = 0; i < 2; ++i) {
        if (c->tab_host[i]) hipHostFree(c->tab_host[i]);
        if (c->tab_ev[i]) hipEventDestroy(c->tab_ev[i]);
    }
    if (c->ban_host) hipHostFree(c->ban_host);
    for (int i = 0; i < asynclm_ctx::BAN_RING; ++i)
        if (c->ban_ev[i]) hipEventDestroy(c->ban_ev[i]);
    delete c;
    return ASYNCLM_OK;
}

int asynclm_prefill(asynclm_ctx* c, int32_t seq, const int32_t* tokens, int32_t n) {
    int r = check_seq(c, seq);
    if (r) return r;
    if ((r = check_tokens(c, tokens, n))) return r;
    if (c->len[seq] != 0) return ASYNCLM_E_STATE;
    if (n > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
    return append_tokens(c, seq, tokens, n);
}

int asynclm_decode_step(asynclm_ctx* c, int32_t seq, int32_t forced_token, int32_t* token_out) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (forced_token >= c->cfg.vocab) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    if (c->len[seq] + 1 > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
    HIPCK(c, step_one_token(c, seq, forced_token < 0 ? -1 : forced_token, true));
    if (token_out) {
        if (c->tok_early) {                         // per-operation step: wait for the choice only
            HIPCK(c, hipEventSynchronize(c->tok_event));
            *token_out = c->token_host[4];
            return ASYNCLM_OK;
        }
        HIPCK(c, hipMemcpyAsync(c->token_host, c->b.token_log, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        HIPCK(c, hipStreamSynchronize(c->stream));
        if (c->token_host[1]) return fail_device(c, hipErrorLaunchFailure);
        *token_out = c->token_host[0];
    }
    return ASYNCLM_OK;
}

int asynclm_inject_interrupt(asynclm_ctx* c, int32_t seq, const int32_t* tokens, int32_t k) {
    int r = check_seq(c, seq);
    if (r) return r;
    if ((r = check_tokens(c, tokens, k))) return r;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    if ((int64_t)c->len[seq] + k > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
    return append_tokens(c, seq, tokens, k);
}

int asynclm_step_batch(asynclm_ctx* c, int32_t nseq, const int32_t* seqs, const int32_t* forced, const int32_t* intr_tokens,
                       const int32_t* intr_offsets, int32_t* tokens_out) {
    if (!c) return ASYNCLM_E_INVAL;
    if (c->poisoned) return ASYNCLM_E_DEVICE;
    if (nseq < 1 || nseq > c->cfg.max_seqs || !seqs) return ASYNCLM_E_INVAL;
    // everything is checked before anything is enqueued
    {
        std::vector<char>& seen = c->batch_seen;
        std::fill(seen.begin(), seen.end(), 0);
        for (int i = 0; i < nseq; ++i) {
            const int q = seqs[i];
            if (q < 0 || q >= c->cfg.max_seqs || seen[q]) return ASYNCLM_E_INVAL;
            seen[q] = 1;
            if (forced && forced[i] >= c->cfg.vocab) return ASYNCLM_E_INVAL;
            if (intr_offsets && intr_offsets[i + 1] < intr_offsets[i]) return ASYNCLM_E_INVAL;
        }
        if (intr_offsets && intr_offsets[0] < 0) return ASYNCLM_E_INVAL;
        if (intr_offsets && intr_offsets[nseq] > intr_offsets[0] && !intr_tokens) return ASYNCLM_E_INVAL;
        if (intr_offsets)
            for (int j = intr_offsets[0]; j < intr_offsets[nseq]; ++j)
                if (intr_tokens[j] < 0 || intr_tokens[j] >= c->cfg.vocab) return ASYNCLM_E_INVAL;
        for (int i = 0; i < nseq; ++i)
            if (c->len[seqs[i]] == 0) return ASYNCLM_E_STATE;
        for (int i = 0; i < nseq; ++i) {
            const int64_t k = intr_offsets ? intr_offsets[i + 1] - intr_offsets[i] : 0;
            if ((int64_t)c->len[seqs[i]] + 1 + k > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
        }
    }
    auto forced_of = [&](int i) { return forced && forced[i] >= 0 ? forced[i] : -1; };
    if (nseq == 1 && (!intr_offsets || intr_offsets[1] == intr_offsets[0]))
        return asynclm_decode_step(c, seqs[0], forced_of(0), tokens_out);      // one row: the single-row kernels

    if (!c->chunk_ok) {
        // models outside the matrix-core append path: the same result sequence by sequence through the single-row kernels
        for (int i = 0; i < nseq; ++i) {
            const int k = intr_offsets ? intr_offsets[i + 1] - intr_offsets[i] : 0;
            HIPCK(c, step_one_token(c, seqs[i], forced_of(i), k == 0));
            if (tokens_out) {
                HIPCK(c, hipMemcpyAsync(c->token_host, c->b.token_log, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
                HIPCK(c, hipStreamSynchronize(c->stream));
                if (c->token_host[1]) return fail_device(c, hipErrorLaunchFailure);
                tokens_out[i] = c->token_host[0];
            }
            if (k > 0) {
                const int r = append_tokens(c, seqs[i], intr_tokens + intr_offsets[i], k);
                if (r) return r;
            }
        }
        return ASYNCLM_OK;
    }

    // One weight pass per CHUNK_MAX rows: groups are packed in the order given; a group that does not fit is
    // continued in the next pass (its later rows see its earlier ones through the cache).
    for (int i = 0; i < nseq; ++i)
        if (forced_of(i) < 0) HIPCK(c, refresh_choice(c, seqs[i]));
    PassBuilder& pb = c->pass;
    std::vector<int>& owner = c->batch_owner;   // group of the current pass -> index i whose token it chooses, or -1
    owner.clear();
    auto flush = [&]() -> int {
        if (pb.t.rows == 0) return ASYNCLM_OK;
        const int ng = pb.t.ngroups;
        HIPCK(c, forward_chunk(c, pb));
        if (tokens_out) {
            HIPCK(c, hipMemcpyAsync(c->chosen_host, c->cb.chosen, sizeof(int32_t) * ng, hipMemcpyDeviceToHost, c->stream));
            HIPCK(c, hipStreamSynchronize(c->stream));
            for (int gi = 0; gi < ng; ++gi)
                if (owner[gi] >= 0) tokens_out[owner[gi]] = c->chosen_host[gi];
        }
        pb.clear();
        owner.clear();
        return ASYNCLM_OK;
    };
    pb.clear();
    for (int i = 0; i < nseq; ++i) {
        const int q = seqs[i];
        const int k = intr_offsets ? intr_offsets[i + 1] - intr_offsets[i] : 0;
        const int32_t* it = k ? intr_tokens + intr_offsets[i] : nullptr;
        int done = 0;                       // rows of this sequence already placed (the chosen token is row 0)
        const int total = 1 + k;
        while (done < total) {
            int space = CHUNK_MAX - pb.t.rows;
            if (space == 0 || !pb.fits(1)) { const int r = flush(); if (r) return r; space = CHUNK_MAX; }
            int n = std::min(space, total - done);
            while (n > 1 && !pb.fits(n)) --n;
            const int pos0 = c->len[q];     // rows placed by earlier passes are already counted
            if (done == 0) pb.add(q, pos0, n, forced_of(i), it, done + n == total);
            else pb.add(q, pos0, n, -2, it + (done - 1), done + n == total);
            owner.push_back(done == 0 ? i : -1);
            done += n;
            if (done < total) { const int r = flush(); if (r) return r; }
        }
    }
    return flush();
}

int asynclm_set_banned_tokens(asynclm_ctx* c, int32_t seq, const int32_t* ids, int32_t n) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (n < 0 || n > BAN_MAX || (n > 0 && !ids)) return ASYNCLM_E_INVAL;
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= c->cfg.vocab) return ASYNCLM_E_INVAL;
    // through a pinned row (asynchronous copy; stream order puts it before later steps)
    const int slot = c->ban_next;
    HIPCK(c, hipEventSynchronize(c->ban_ev[slot]));
    int32_t* row = c->ban_host + (size_t)slot * (1 + BAN_MAX);
    std::memset(row, 0, sizeof(int32_t) * (1 + BAN_MAX));
    row[0] = n;
    for (int i = 0; i < n; ++i) row[1 + i] = ids[i];
    HIPCK(c, hipMemcpyAsync(c->b.banned + (size_t)seq * (1 + BAN_MAX), row, sizeof(int32_t) * (1 + BAN_MAX), hipMemcpyHostToDevice, c->stream));
    HIPCK(c, hipEventRecord(c->ban_ev[slot], c->stream));
    c->ban_next = (slot + 1) % asynclm_ctx::BAN_RING;
    c->nban[seq] = n;
    if (c->len[seq] > 0) c->choice_stale[seq] = 1;      // the next greedy choice is recomputed under the new list
    return ASYNCLM_OK;
}

// ---- K/V swap (trap handling) ---------------------------------------------------------------------------------

namespace {

struct SwapHeader {
    uint32_t magic, version;
    int32_t len, n_layers, n_planes, has_vt, elem_bytes, Hkv, dh, vocab, next_token, pad;
    uint64_t total_bytes;
};
constexpr uint32_t SWAP_MAGIC = 0x4b56414cu;     // "LAVK"

int swap_planes(const asynclm_ctx* c) {          // row-major planes per layer: K (+lo), and V (+lo) where it is kept
    return (c->g.kv_lo_offset ? 2 : 1) * (c->g.kv_v_offset ? 2 : 1);
}

size_t swap_bytes(const asynclm_ctx* c, int len) {
    const Geom& g = c->g;
    const size_t esz = elem_bytes(c);
    const size_t rows = (size_t)len * g.dh * g.Hkv * esz;                                  // one row-major plane
    const size_t vt = g.kv_vt_offset ? (size_t)((len + 31) / 32) * 32 * g.dh * g.Hkv * esz : 0;   // one tiled V^T plane
    return sizeof(SwapHeader) + (size_t)c->cfg.n_layers * (swap_planes(c) * rows + 2 * vt) + (size_t)g.V * sizeof(float);
}

// Copies every cached row of `seq` between the cache and the packed host image (direction by `out`).
hipError_t swap_copy(asynclm_ctx* c, int seq, int len, char* host, bool out) {
    const Geom& g = c->g;
    const size_t esz = elem_bytes(c);
    const size_t width = (size_t)len * g.dh * esz, pitch = g.kv_head_stride * esz;
    const size_t vt_width = (size_t)((len + 31) / 32) * 32 * g.dh * esz;
    const hipMemcpyKind kind = out ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice;
    char* h = host;
    hipError_t e;
    for (int l = 0; l < c->cfg.n_layers; ++l) {
        char* base = (char*)kv_layer_ptr(c, l) + (size_t)seq * g.kv_seq_stride * esz;
        size_t offs[4]; int np = 0;
        offs[np++] = 0;
        if (g.kv_lo_offset) offs[np++] = g.kv_lo_offset;
        if (g.kv_v_offset) {
            offs[np++] = g.kv_v_offset;
            if (g.kv_lo_offset) offs[np++] = g.kv_v_offset + g.kv_lo_offset;
        }
        for (int p = 0; p < np; ++p) {
            char* dev = base + offs[p] * esz;
            e = out ? hipMemcpy2DAsync(h, width, dev, pitch, width, g.Hkv, kind, c->stream)
                    : hipMemcpy2DAsync(dev, pitch, h, width, width, g.Hkv, kind, c->stream);
            if (e) return e;
            h += width * g.Hkv;
        }
        if (g.kv_vt_offset) {
            for (int p = 0; p < 2; ++p) {
                char* dev = base + (g.kv_vt_offset + (p ? g.kv_lo_offset : 0)) * esz;
                e = out ? hipMemcpy2DAsync(h, vt_width, dev, pitch, vt_width, g.Hkv, kind, c->stream)
                        : hipMemcpy2DAsync(dev, pitch, h, vt_width, vt_width, g.Hkv, kind, c->stream);
                if (e) return e;
                h += vt_width * g.Hkv;
            }
        }
    }
    float* lg = c->logits + (size_t)seq * g.V;
    e = out ? hipMemcpyAsync(h, lg, sizeof(float) * g.V, kind, c->stream) : hipMemcpyAsync(lg, h, sizeof(float) * g.V, kind, c->stream);
    return e;
}

}  // namespace

int asynclm_kv_bytes(asynclm_ctx* c, int32_t seq, uint64_t* bytes) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!bytes) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    *bytes = swap_bytes(c, c->len[seq]);
    return ASYNCLM_OK;
}

int asynclm_kv_swap_out(asynclm_ctx* c, int32_t seq, void* host_buf, uint64_t capacity) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!host_buf) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    const int len = c->len[seq];
    const size_t need = swap_bytes(c, len);
    if (capacity < need) return ASYNCLM_E_CAPACITY;
    HIPCK(c, refresh_choice(c, seq));           // the saved greedy token is the one under the current ban list
    SwapHeader hd{};
    hd.magic = SWAP_MAGIC; hd.version = 1; hd.len = len; hd.n_layers = c->cfg.n_layers; hd.n_planes = swap_planes(c);
    hd.has_vt = c->g.kv_vt_offset ? 1 : 0; hd.elem_bytes = (int32_t)elem_bytes(c); hd.Hkv = c->g.Hkv; hd.dh = c->g.dh;
    hd.vocab = c->g.V; hd.total_bytes = need;
    HIPCK(c, swap_copy(c, seq, len, (char*)host_buf + sizeof(SwapHeader), true));
    HIPCK(c, hipMemcpyAsync(c->token_host, &c->b.seq_state[seq].next_token, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIPCK(c, hipStreamSynchronize(c->stream));
    hd.next_token = c->token_host[0];
    std::memcpy(host_buf, &hd, sizeof(hd));
    return ASYNCLM_OK;
}

int asynclm_kv_swap_in(asynclm_ctx* c, int32_t seq, const void* host_buf, uint64_t bytes) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!host_buf || bytes < sizeof(SwapHeader)) return ASYNCLM_E_INVAL;
    if (c->len[seq] != 0) return ASYNCLM_E_STATE;
    SwapHeader hd;
    std::memcpy(&hd, host_buf, sizeof(hd));
    if (hd.magic != SWAP_MAGIC || hd.version != 1 || hd.len < 1 || hd.n_layers != c->cfg.n_layers || hd.n_planes != swap_planes(c) ||
        hd.has_vt != (c->g.kv_vt_offset ? 1 : 0) || hd.elem_bytes != (int32_t)elem_bytes(c) || hd.Hkv != c->g.Hkv || hd.dh != c->g.dh ||
        hd.vocab != c->g.V || hd.next_token < 0 || hd.next_token >= c->g.V)
        return ASYNCLM_E_INVAL;
    if (hd.len > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
    if (hd.total_bytes != swap_bytes(c, hd.len) || bytes < hd.total_bytes) return ASYNCLM_E_INVAL;
    HIPCK(c, swap_copy(c, seq, hd.len, (char*)const_cast<void*>(host_buf) + sizeof(SwapHeader), false));
    SeqState st{hd.len, hd.next_token};
    HIPCK(c, hipMemcpyAsync(c->b.seq_state + seq, &st, sizeof(st), hipMemcpyHostToDevice, c->stream));
    HIPCK(c, hipStreamSynchronize(c->stream));   // the host image may be released when the call returns
    c->len[seq] = hd.len;
    c->choice_stale[seq] = c->nban[seq] > 0;     // the restored token was chosen under the saver's list
    return ASYNCLM_OK;
}

int asynclm_peek_token(asynclm_ctx* c, int32_t seq, int32_t* token_out) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!token_out) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    HIPCK(c, refresh_choice(c, seq));
    HIPCK(c, hipMemcpyAsync(c->token_host, &c->b.seq_state[seq].next_token, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIPCK(c, hipStreamSynchronize(c->stream));
    *token_out = c->token_host[0];
    return ASYNCLM_OK;
}

int asynclm_logits(asynclm_ctx* c, int32_t seq, float* out_host, int32_t n) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!out_host || n != c->cfg.vocab) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    HIPCK(c, hipMemcpyAsync(out_host, c->logits + (size_t)seq * c->g.V, sizeof(float) * n, hipMemcpyDeviceToHost, c->stream));
    HIPCK(c, hipMemcpyAsync(c->token_host, c->b.token_log, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIPCK(c, hipStreamSynchronize(c->stream));
    if (c->token_host[1]) return fail_device(c, hipErrorLaunchFailure);
    return ASYNCLM_OK;
}

int asynclm_logits_device(asynclm_ctx* c, int32_t seq, const float** out_dev) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!out_dev) return ASYNCLM_E_INVAL;
    *out_dev = c->logits + (size_t)seq * c->g.V;
    return ASYNCLM_OK;
}

int asynclm_seq_len(asynclm_ctx* c, int32_t seq, int32_t* len) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!len) return ASYNCLM_E_INVAL;
    *len = c->len[seq];
    return ASYNCLM_OK;
}

int asynclm_reset(asynclm_ctx* c, int32_t seq) {
    int r = check_seq(c, seq);
    if (r) return r;
    HIPCK(c, hipMemsetAsync(c->b.seq_state + seq, 0, sizeof(SeqState), c->stream));
    c->len[seq] = 0;
    c->choice_stale[seq] = 0;
    return ASYNCLM_OK;
}

int asynclm_synchronize(asynclm_ctx* c) {
    if (!c) return ASYNCLM_E_INVAL;
    if (c->poisoned) return ASYNCLM_E_DEVICE;
    HIPCK(c, hipStreamSynchronize(c->stream));
    return ASYNCLM_OK;
}

int asynclm_set_option(asynclm_ctx* c, const char* name, int32_t value) {
    if (!c || !name) return ASYNCLM_E_INVAL;
    if (!std::strcmp(name, "chunk")) { if (value < 1 || value > CHUNK_MAX) return ASYNCLM_E_INVAL; c->opt_chunk = value; return ASYNCLM_OK; }
    if (!std::strcmp(name, "chunk_split")) { if (value < 0 || value > CHUNK_GEMM_MAX_SPLIT) return ASYNCLM_E_INVAL; c->opt_chunk_split = value; return ASYNCLM_OK; }
    // the options below change the launch geometry of a decoding step: its captured graphs are built again (this call allocates)
    auto regraph = [&]() -> int {
        HIPCK(c, hipStreamSynchronize(c->stream));
        HIPCK(c, rebuild_graphs(c));
        return ASYNCLM_OK;
    };
    if (!std::strcmp(name, "gemv_grid")) { if (value < 1 || value > 4096) return ASYNCLM_E_INVAL; decode_set_gemv_grid(value); return regraph(); }
    if (!std::strcmp(name, "fused")) { c->opt_fused = (value && c->fused.supported) ? 1 : 0; return regraph(); }
    if (!std::strcmp(name, "pipeline")) { c->opt_pipeline = (value && c->pipe_ok) ? 1 : 0; return regraph(); }
    if (!std::strcmp(name, "graph")) { c->opt_graph = (value && c->stream) ? 1 : 0; return regraph(); }
    if (!std::strcmp(name, "attn_mfma_min")) { if (value < 0) return ASYNCLM_E_INVAL; c->opt_attn_mfma_min = value; return regraph(); }
    if (!std::strcmp(name, "step_stamps")) { c->opt_step_stamps = value ? 1 : 0; return regraph(); }
    if (!std::strcmp(name, "attn_split")) { if (value < 0 || value > CHUNK_ATTN_MAX_SPLIT) return ASYNCLM_E_INVAL; c->opt_attn_split = value; return regraph(); }
    return ASYNCLM_E_INVAL;
}

int asynclm_profile_step(asynclm_ctx* c, int32_t seq, int32_t forced_token, const char* const** names_out,
                         float* ms_out, int32_t* launches_out, int32_t cap) {
    int r = check_seq(c, seq);
    if (r) return r;
    if (!ms_out || !launches_out || cap < KC_COUNT || forced_token < 0 || forced_token >= c->cfg.vocab) return ASYNCLM_E_INVAL;
    if (c->len[seq] == 0) return ASYNCLM_E_STATE;
    if (c->len[seq] + 1 > c->cfg.max_positions) return ASYNCLM_E_CAPACITY;
    for (hipEvent_t ev : c->prof_events) hipEventDestroy(ev);
    c->prof_events.clear(); c->prof_class.clear();
    for (int i = 0; i < KC_COUNT; ++i) { ms_out[i] = 0.f; launches_out[i] = 0; }
    if (c->opt_fused) {
        // one launch: HIP events around the kernel, and the kernel's own phase time stamps (100 MHz clock)
        const int nl = c->cfg.n_layers, n_stamps = 1 + 12 * nl + 2;
        if (n_stamps > FUSED_TRACE_MAX) return ASYNCLM_E_INVAL;
        hipEvent_t e0, e1;
        HIPCK(c, hipEventCreate(&e0)); HIPCK(c, hipEventCreate(&e1));
        c->prof_events.push_back(e0); c->prof_events.push_back(e1);
        HIPCK(c, hipEventRecord(e0, c->stream));
        c->want_trace = true;
        hipError_t e = step_one_token(c, seq, forced_token, true);
        c->want_trace = false;
        if (e) return fail_device(c, e);
        HIPCK(c, hipEventRecord(e1, c->stream));
        // stamps [i][workgroup]; a phase lasts from the latest start to the latest finish over the workgroups,
        // a barrier from the latest arrival to the latest release
        const size_t nw = (size_t)c->fused.grid;
        std::vector<unsigned long long> raw((size_t)n_stamps * nw), t(n_stamps);
        HIPCK(c, hipMemcpyAsync(raw.data(), c->trace, sizeof(unsigned long long) * raw.size(), hipMemcpyDeviceToHost, c->stream));
        HIPCK(c, hipStreamSynchronize(c->stream));
        for (int i = 0; i < n_stamps; ++i) t[i] = *std::max_element(raw.begin() + i * nw, raw.begin() + (i + 1) * nw);
        c->last_trace = raw; c->last_trace_stamps = n_stamps;
        float ms = 0.f;
        HIPCK(c, hipEventElapsedTime(&ms, e0, e1));
        ms_out[KC_F_TOTAL] = ms; launches_out[KC_F_TOTAL] = 1;
        auto add = [&](int kc, size_t i) { ms_out[kc] += (float)((double)(t[i] - t[i - 1]) * 1e-5); launches_out[kc] += 1; };
        for (int l = 0; l < nl; ++l) {
            const size_t b = 1 + 12 * (size_t)l;
            for (int k = 0; k < 12; ++k) add(KC_F_QKV + k, b + k);
        }
        add(KC_F_HEAD, 1 + 12 * (size_t)nl); add(KC_F_HEAD_WAIT, 2 + 12 * (size_t)nl);
        if (names_out) *names_out = kClassNames;
        return KC_COUNT;
    }
    c->prof = true;
    hipError_t e = step_one_token(c, seq, forced_token, true);
    c->prof = false;
    if (e) return fail_device(c, e);
    HIPCK(c, hipStreamSynchronize(c->stream));
    for (size_t i = 0; i < c->prof_class.size(); ++i) {
        float ms = 0.f;
        HIPCK(c, hipEventElapsedTime(&ms, c->prof_events[2 * i], c->prof_events[2 * i + 1]));
        ms_out[c->prof_class[i]] += ms;
        launches_out[c->prof_class[i]] += 1;
    }
    if (names_out) *names_out = kClassNames;
    return KC_COUNT;
}

int asynclm_profile_trace(asynclm_ctx* c, uint64_t* out_host, int32_t cap, int32_t* n_stamps, int32_t* n_workgroups) {
    if (!c || !n_stamps || !n_workgroups) return ASYNCLM_E_INVAL;
    if (c->pipe_kernels > 0 && !c->opt_fused) {
        // the last two-stream step (or one-stream step in stamp mode): per kernel, start / hand-over seen (input vector
        // staged) / done of its first and of its last workgroup
        *n_stamps = 3 * c->pipe_kernels; *n_workgroups = 2;
        if (out_host) {
            if (cap < 6 * c->pipe_kernels) return ASYNCLM_E_INVAL;
            std::vector<unsigned long long> raw((size_t)6 * c->pipe_kernels);
            HIPCK(c, hipStreamSynchronize(c->stream));
            HIPCK(c, hipMemcpy(raw.data(), c->pipe_stamps, raw.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
            if (c->last_step_stamp_mode) {      // done: earliest and latest of the workgroups' own words
                std::vector<unsigned long long> done((size_t)c->pipe_kernels * STAMP_DONE_SLOTS);
                HIPCK(c, hipMemcpy(done.data(), c->stamp_done, done.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
                for (int k = 0; k < c->pipe_kernels; ++k) {
                    unsigned long long lo = ~0ull, hi = 0;
                    for (int w = 0; w < STAMP_DONE_SLOTS; ++w) {
                        const unsigned long long t = done[(size_t)k * STAMP_DONE_SLOTS + w];
                        if (t) { lo = std::min(lo, t); hi = std::max(hi, t); }
                    }
                    raw[(size_t)k * 6 + 2] = hi ? lo : 0; raw[(size_t)k * 6 + 5] = hi;
                }
            }
            for (int k = 0; k < c->pipe_kernels; ++k)
                for (int w = 0; w < 2; ++w)
                    for (int j = 0; j < 3; ++j) out_host[(size_t)(3 * k + j) * 2 + w] = raw[(size_t)k * 6 + w * 3 + j];
        }
        return ASYNCLM_OK;
    }
    *n_stamps = c->last_trace_stamps;
    *n_workgroups = c->last_trace_stamps ? (int32_t)(c->last_trace.size() / c->last_trace_stamps) : 0;
    if (out_host) {
        if ((size_t)cap < c->last_trace.size()) return ASYNCLM_E_INVAL;
        for (size_t i = 0; i < c->last_trace.size(); ++i) out_host[i] = c->last_trace[i];
    }
    return ASYNCLM_OK;
}

// ---- greedy choice without any allocation -----------------------------------------------------------------------

namespace {

// Scratch of asynclm_greedy_token_static: per-block maxima, their indices, the arrival counter.  One copy per device
// that loads the library, held until the process ends.  In host code the array's name is not a device address: the
// address comes from hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
struct ArgmaxScratch { float part_v[ARGMAX_MAX_BLOCKS]; int32_t part_i[ARGMAX_MAX_BLOCKS]; int32_t counter; int32_t pad[63]; };
static __device__ __align__(256) unsigned char scratch[sizeof(ArgmaxScratch)];

constexpr int STATIC_MAX_DEVICES = 64;
void* g_scratch_ptr[STATIC_MAX_DEVICES] = {};      // per device: device address of `scratch`

}  // namespace

int asynclm_greedy_token_static(const float* logits_dev, int32_t n, const int32_t* banned_dev, int32_t n_banned,
                                int32_t* token_out_dev, void* hip_stream) {
    if (!logits_dev || !token_out_dev || n < 1 || n > ASYNCLM_STATIC_MAX_VOCAB) return ASYNCLM_E_INVAL;
    if (n_banned < 0 || n_banned > BAN_MAX || (n_banned > 0 && !banned_dev)) return ASYNCLM_E_INVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return ASYNCLM_E_DEVICE;
    if (!g_scratch_ptr[dev]) {          // first call on this device (it is the current one)
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { report_hip("hipGetSymbolAddress", e); return ASYNCLM_E_DEVICE; }
        g_scratch_ptr[dev] = p;
    }
    ArgmaxScratch* sc = (ArgmaxScratch*)g_scratch_ptr[dev];
    const hipError_t e = launch_argmax_flat(logits_dev, n, banned_dev, n_banned, sc->part_v, sc->part_i, &sc->counter, token_out_dev,
                                            (hipStream_t)hip_stream);
    if (e != hipSuccess) { report_hip("asynclm_greedy_token_static", e); return ASYNCLM_E_DEVICE; }
    return ASYNCLM_OK;
}

const char* asynclm_strerror(int code) {
    switch (code) {
        case ASYNCLM_OK: return "ok";
        case ASYNCLM_E_INVAL: return "invalid argument";
        case ASYNCLM_E_STATE: return "call not allowed in this sequence state";
        case ASYNCLM_E_CAPACITY: return "sequence would exceed max_positions";
        case ASYNCLM_E_NOMEM: return "out of memory";
        case ASYNCLM_E_DEVICE: return "HIP error (context unusable)";
        default: return "unknown error";
    }
}

const char* asynclm_version(void) { return "0.1.0"; }

}  // extern "C"
