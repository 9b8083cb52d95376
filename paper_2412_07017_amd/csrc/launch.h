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

hipError_t decode_init(int dtype, int max_k);
hipError_t launch_begin_step(const DecodeBuffers& b, int seq, int forced, hipStream_t s);
hipError_t launch_embed(int dtype, const void* E, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_qkv(int dtype, const void* wqkv, const float* gain, void* kv_layer, const DecodeBuffers& b,
                      const Geom& g, hipStream_t s);
hipError_t launch_attn_decode(int dtype, const void* kv_layer, int nsplit, const DecodeBuffers& b, const Geom& g,
                              hipStream_t s);
hipError_t launch_oproj(int dtype, const void* wo, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_gateup(int dtype, const void* wgu, const float* gain, const DecodeBuffers& b, const Geom& g,
                         hipStream_t s);
hipError_t launch_down(int dtype, const void* wd, const DecodeBuffers& b, const Geom& g, hipStream_t s);
hipError_t launch_lmhead(int dtype, const void* wout, const float* gain, float* logits, const DecodeBuffers& b,
                         const Geom& g, hipStream_t s);
hipError_t launch_argmax(const float* logits_base, const DecodeBuffers& b, const Geom& g, hipStream_t s);

}  // namespace asynclm
