// Host-callable launchers of the device code (one function per kernel class).
#pragma once

#include "common.h"

namespace asynclm {

constexpr int ARGMAX_MAX_BLOCKS = 256;
constexpr int BAN_MAX = 31;            // token ids per sequence that the greedy choice may be told to skip
constexpr int ATTN_MAX_SPLIT = 64;

// Device buffers of the single-row (decode) path.  All fp32 unless noted.
struct DecodeBuffers {
    StepDesc* step;
    SeqState* seq_state;      // [max_seqs]
    int32_t* token_log;       // last token chosen by k_begin_step
    float* x;                 // [d] residual stream
    float* x2;                // [d] residual stream after the attention block (two-stream step only)
    float* q;                 // [Hq*dh]
    float* o;                 // [Hq*dh]
    float* a;                 // [F]
    float* part_acc;          // [Hq][ATTN_MAX_SPLIT][dh]
    float* part_ml;           // [Hq][ATTN_MAX_SPLIT][2]
    int32_t* attn_counters;   // [Hkv]
    float* amax_v;            // [ARGMAX_MAX_BLOCKS]
    int32_t* amax_i;
    int32_t* amax_counter;
    int32_t* banned;          // [max_seqs][1 + BAN_MAX]: count, then the ids the greedy choice of the sequence skips
    const float* rope_cos;    // [max_pos][dh/2]
    const float* rope_sin;
    unsigned* pipe_abort;     // give-up word of the two-stream step (see PipeSync)
};

constexpr int CHUNK_MAX = 512;         // rows per forward pass of the append-chunk path
constexpr int CHUNK_MAX_TASKS = 128;   // attention tiles (32 query columns of one group) per pass
constexpr int CHUNK_ATTN_MAX_SPLIT = 128;
constexpr int CHUNK_ATTN_MAX_UNITS = 4096;   // (task, kv head, key split) partial results per pass
constexpr int CHUNK_GEMM_MAX_SPLIT = 8;

// What one pass of the append-chunk path processes: rows, grouped by sequence.  A group is a run of
// consecutive rows appended to one sequence: [chosen token] ++ [interrupt tokens], or plain tokens.
// The host fills the table; k_begin_chunk resolves the tokens that are chosen on the device.
struct ChunkRow { int32_t token, seq, pos, row0, n, pad0, pad1, pad2; };          // row0, n: its group
struct ChunkGroup {
    int32_t seq, row0, n, pos0;
    int32_t forced;     // first row: >= 0 this token, -1 greedy argmax of the sequence's logits, -2 already in the row table
    int32_t head;       // row of this group in the output-head product, -1: no logits wanted
    int32_t pad0, pad1;
};
struct ChunkTask { int32_t seq, row0, n, pos0, tile, pad0, pad1, pad2; };         // query columns 32 tile .. 32 tile + 31 of a group
// Every group has at least one task, so a pass holds at most CHUNK_MAX_TASKS groups.  The rows come last: a
// pass uploads the table up to its last used row.
struct ChunkTaskBlock { int32_t task0, n; };   // up to four consecutive tasks of one group (they share keys and values)
struct ChunkTable {
    int32_t rows, ngroups, ntasks, nhead;
    int32_t nblocks, pad0, pad1, pad2;
    ChunkGroup group[CHUNK_MAX_TASKS];
    ChunkTask task[CHUNK_MAX_TASKS];
    ChunkTaskBlock block[CHUNK_MAX_TASKS];
    ChunkRow row[CHUNK_MAX];
};

// Device buffers of the append-chunk path (bf16 models).  "hi/lo" are the two bf16 planes of a value.
struct ChunkBuffers {
    ChunkTable* tab;
    int32_t* chosen;          // [CHUNK_MAX] token chosen for the first row of each group
    float* x;                 // [CHUNK_MAX][d] residual stream
    // inputs of the products, CHUNK_MAX rows each, stored in matrix-core operand order (tiled planes)
    bf16_t *nrm_hi, *nrm_lo;  // d columns:     normalised input of the QKV, gate/up and output-head products
    bf16_t *att_hi, *att_lo;  // Hq*dh columns: attention output
    bf16_t *act_hi, *act_lo;  // F columns:     SwiGLU output
    // rotated, scaled queries [Hkv][q_cols][dh]: the columns of a group are [q head within the kv group][row]
    bf16_t *q_hi, *q_lo;
    int q_cols;               // G * CHUNK_MAX + 32 (a tile may read up to 31 columns past its group)
    float* part;              // split-K partial planes of the current product
    size_t part_capacity;     // floats in `part`
    float* attn_o;            // [unit][dh][32]      unit = (task * Hkv + kv head) * nsplit + split
    float* attn_ml;           // [unit][2][32]
};

// Fused (persistent, single-kernel) decoding step.
struct FusedPlan {
    bool supported;
    int grid;           // workgroups = compute units
    int nsplit;         // largest number of attention splits per kv head
    int xs_groups;      // LDS capacity of the staged vector
    int done_cap;       // finished units a wave can park in LDS
    size_t lds_bytes;
};
struct FusedLaunch {
    const void* layers_dev;     // device array, 7 pointers per layer: attn_norm, wqkv, wo, ffn_norm, wgate_up, wdown, kv_layer
    int n_layers;
    const void* embed; const float* final_norm; const void* lm_head;
    int seq, forced; bool with_head;
    int nsplit; bool merge_in_stage;   // attention splits of this step; merged by the O projection's staging if set
    float* logits;              // of this sequence
    unsigned* bar;              // FUSED_BAR_WORDS words, zero at create
    void* trace;                // optional device buffer of 64-bit time stamps [FUSED_TRACE_MAX][grid]
};
constexpr int FUSED_TRACE_MAX = 4096;
constexpr int FUSED_BAR_WORDS = 8 + 1024;   // barrier header + one flag per workgroup
hipError_t fused_init(int dtype, const Geom& g, FusedPlan* plan);
hipError_t launch_decode_fused(int dtype, const FusedPlan& plan, const FusedLaunch& L, const DecodeBuffers& b, const Geom& g,
                               hipStream_t s);

hipError_t decode_init(int dtype, int max_k);
void decode_set_gemv_grid(int grid);
int decode_gemv_grid();
hipError_t chunk_init();
hipError_t launch_begin_chunk(const ChunkBuffers& c, const DecodeBuffers& b, int ngroups, hipStream_t s);
hipError_t launch_chunk_embed(const void* E, const ChunkBuffers& c, int rows, const Geom& g, hipStream_t s);
hipError_t launch_chunk_resid_norm(const ChunkBuffers& c, bool add_partials, int S, int MT, const float* gain, int rows,
                                   const Geom& g, hipStream_t s);
// residual stream of the last row of group `group` -> the single-row path's x (and its sequence -> the step descriptor)
hipError_t launch_chunk_last_row(const ChunkBuffers& c, int S, int MT, int group, const DecodeBuffers& b, const Geom& g,
                                 hipStream_t s);
// last rows of all groups that want logits: residual + final norm -> rows 0..nhead-1 of the nrm planes
hipError_t launch_chunk_head_rows(const ChunkBuffers& c, int S, int MT, const float* gain, int ngroups, const Geom& g,
                                  hipStream_t s);
// rows of the head product -> logits of their sequences, greedy argmax -> next_token
hipError_t launch_chunk_logits(const ChunkBuffers& c, int MT_head, float* logits_base, const DecodeBuffers& b, int ngroups,
                               const Geom& g, hipStream_t s);
hipError_t launch_chunk_swiglu(const ChunkBuffers& c, int S, int MT, int rows, const Geom& g, hipStream_t s);
hipError_t launch_chunk_rope_kv(const ChunkBuffers& c, int S, void* kv_layer, const DecodeBuffers& b, int rows, int MT,
                                const Geom& g, hipStream_t s);
hipError_t launch_chunk_gemm(const void* W, int N, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                             int S, int MT, hipStream_t s);
hipError_t launch_chunk_gemm_swiglu(const void* W, int F, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                                    int MT, hipStream_t s);
hipError_t launch_chunk_attn(const ChunkBuffers& c, const void* kv_layer, int nsplit, int ntasks, const Geom& g, hipStream_t s);
hipError_t launch_chunk_attn_wide(const ChunkBuffers& c, const void* kv_layer, int nsplit, int ntasks, int nblocks, const Geom& g,
                                  hipStream_t s);
// single-row decoding attention on the matrix cores (long contexts): b.q -> b.o through the chunk attention
// stamps / done_wg: null, or the stamp words (2 x 6) and finishing-time words (2 x STAMP_DONE_SLOTS) of the attention
// kernel and of its merge kernel (see step_stamp_done)
hipError_t launch_decode_attn_mfma(const ChunkBuffers& c, const void* kv_layer, int nsplit, const DecodeBuffers& b, const Geom& g,
                                   hipStream_t s, unsigned long long* stamps = nullptr, unsigned long long* done_wg = nullptr);
hipError_t launch_stamp_init(unsigned long long* done_wg, int kernels, hipStream_t s);
// token_early: pinned host word that also gets the chosen token (or nullptr)
hipError_t launch_begin_step(const DecodeBuffers& b, int seq, int forced, int32_t* token_early, hipStream_t s);
hipError_t launch_embed(int dtype, const void* E, const DecodeBuffers& b, const Geom& g, hipStream_t s);
// sync (all single-row launchers): hand-over flags when the step's kernels alternate between two streams (see PipeSync)
hipError_t launch_qkv(int dtype, const void* wqkv, const float* gain, void* kv_layer, const DecodeBuffers& b,
                      const Geom& g, hipStream_t s, const PipeSync* sync = nullptr);
// merge_in_oproj: the attention only leaves per-split partials and the O projection merges them (nsplit <= 8)
hipError_t launch_attn_decode(int dtype, const void* kv_layer, int nsplit, bool merge_in_oproj, const DecodeBuffers& b,
                              const Geom& g, hipStream_t s, const PipeSync* sync = nullptr);
// x_out / x_in / res_in: the residual stream between the O projection and the down projection lives in a second
// vector when given (the two-stream step never updates a vector in place); default: b.x throughout
hipError_t launch_oproj(int dtype, const void* wo, int merge_nsplit, const DecodeBuffers& b, const Geom& g, hipStream_t s,
                        const PipeSync* sync = nullptr, float* x_out = nullptr);
hipError_t launch_gateup(int dtype, const void* wgu, const float* gain, const DecodeBuffers& b, const Geom& g,
                         hipStream_t s, const PipeSync* sync = nullptr, const float* x_in = nullptr);
hipError_t launch_down(int dtype, const void* wd, const DecodeBuffers& b, const Geom& g, hipStream_t s, const PipeSync* sync = nullptr,
                       const float* res_in = nullptr);
// logits_base: [sequences][V]; the kernel writes the row of the step descriptor's sequence
hipError_t launch_lmhead(int dtype, const void* wout, const float* gain, float* logits_base, const DecodeBuffers& b,
                         const Geom& g, hipStream_t s, const PipeSync* sync = nullptr);
// True when two workgroups of every single-row kernel of this model fit one compute unit (registers, LDS), i.e. when
// the workgroups of two neighbouring kernels of a step can always all be resident: the condition for running the
// step on two streams.
bool decode_pipeline_fits(int dtype, const Geom& g, bool kv_pair);
// greedy choice (banned ids skipped) of sequence `seq`, or of the step descriptor's sequence when seq < 0
hipError_t launch_argmax(const float* logits_base, const DecodeBuffers& b, const Geom& g, hipStream_t s, int seq = -1);
// the same choice over caller-provided logits[n], skipping the nban ids in ban; part_v / part_i: ARGMAX_MAX_BLOCKS entries
// of scratch, counter: one word of scratch (cleared by the launch); the result goes to *out (device)
hipError_t launch_argmax_flat(const float* logits, int n, const int32_t* ban, int nban, float* part_v, int32_t* part_i,
                              int32_t* counter, int32_t* out, hipStream_t s);

}  // namespace asynclm
