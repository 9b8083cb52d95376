// Host-callable launchers of the device code (one function per kernel class).
#pragma once

#include "common.h"

namespace asynclm {

constexpr int ARGMAX_MAX_BLOCKS = 256;
constexpr int ATTN_MAX_SPLIT = 64;

// Device buffers of the single-row (decode) path.  All fp32 unless noted.
struct DecodeBuffers {
    StepDesc* step;
    SeqState* seq_state;      // [max_seqs]
    int32_t* token_log;       // last token chosen by k_begin_step
    float* x;                 // [d] residual stream
    float* q;                 // [Hq*dh]
    float* o;                 // [Hq*dh]
    float* a;                 // [F]
    float* part_acc;          // [Hq][ATTN_MAX_SPLIT][dh]
    float* part_ml;           // [Hq][ATTN_MAX_SPLIT][2]
    int32_t* attn_counters;   // [Hkv]
    float* amax_v;            // [ARGMAX_MAX_BLOCKS]
    int32_t* amax_i;
    int32_t* amax_counter;
    const float* rope_cos;    // [max_pos][dh/2]
    const float* rope_sin;
};

constexpr int CHUNK_MAX = 64;          // rows per forward pass of the append-chunk path
constexpr int CHUNK_ATTN_MAX_SPLIT = 32;
constexpr int CHUNK_GEMM_MAX_SPLIT = 4;

// Device buffers of the append-chunk path (bf16 models).  "hi/lo" are the two bf16 planes of a value.
struct ChunkBuffers {
    int32_t* tokens;          // [CHUNK_MAX]
    float* x;                 // [CHUNK_MAX][d] residual stream
    // inputs of the products, CHUNK_MAX rows each, stored in matrix-core operand order (tiled planes)
    bf16_t *nrm_hi, *nrm_lo;  // d columns:     normalised input of the QKV and gate/up products
    bf16_t *att_hi, *att_lo;  // Hq*dh columns: attention output
    bf16_t *act_hi, *act_lo;  // F columns:     SwiGLU output
    bf16_t *q_hi, *q_lo;      // [Hq][CHUNK_MAX][dh] rotated, scaled queries
    float* part;              // split-K partial planes of the current product
    size_t part_capacity;     // floats in `part`
    float* attn_o;            // [tasks][split][dh][32]
    float* attn_ml;           // [tasks][split][2][32]
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
hipError_t launch_begin_chunk(const DecodeBuffers& b, int seq, int rows, hipStream_t s);
hipError_t launch_chunk_embed(const void* E, const ChunkBuffers& c, int rows, const Geom& g, hipStream_t s);
hipError_t launch_chunk_resid_norm(const ChunkBuffers& c, bool add_partials, int S, int MT, const float* gain, int rows,
                                   const Geom& g, hipStream_t s);
hipError_t launch_chunk_last_row(const ChunkBuffers& c, int S, int MT, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_chunk_swiglu(const ChunkBuffers& c, int S, int MT, int rows, const Geom& g, hipStream_t s);
hipError_t launch_chunk_rope_kv(const ChunkBuffers& c, int S, void* kv_layer, const DecodeBuffers& b, int rows, int MT,
                                const Geom& g, hipStream_t s);
hipError_t launch_chunk_gemm(const void* W, int N, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                             int S, int MT, hipStream_t s);
hipError_t launch_chunk_attn(const ChunkBuffers& c, const void* kv_layer, int nsplit, int MT, const DecodeBuffers& b,
                             const Geom& g, hipStream_t s);
hipError_t launch_begin_step(const DecodeBuffers& b, int seq, int forced, hipStream_t s);
hipError_t launch_embed(int dtype, const void* E, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_qkv(int dtype, const void* wqkv, const float* gain, void* kv_layer, const DecodeBuffers& b,
                      const Geom& g, hipStream_t s);
// merge_in_oproj: the attention only leaves per-split partials and the O projection merges them (nsplit <= 8)
hipError_t launch_attn_decode(int dtype, const void* kv_layer, int nsplit, bool merge_in_oproj, const DecodeBuffers& b,
                              const Geom& g, hipStream_t s);
hipError_t launch_oproj(int dtype, const void* wo, int merge_nsplit, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_gateup(int dtype, const void* wgu, const float* gain, const DecodeBuffers& b, const Geom& g,
                         hipStream_t s);
hipError_t launch_down(int dtype, const void* wd, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_lmhead(int dtype, const void* wout, const float* gain, float* logits, const DecodeBuffers& b,
                         const Geom& g, hipStream_t s);
hipError_t launch_argmax(const float* logits_base, const DecodeBuffers& b, const Geom& g, hipStream_t s);

}  // namespace asynclm
