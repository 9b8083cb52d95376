// Shared declarations of the library's translation units (host + device).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace asynclm {

typedef uint16_t bf16_t;   // raw bfloat16 bits

// Per-launch descriptor living in device memory.  Kernels read the token, its position and the
// sequence from here, so the launch parameters of a decoding step never change and the whole
// step can be replayed as a captured graph.
struct StepDesc {
    int32_t token;   // token processed by this forward pass (decode path)
    int32_t pos;     // absolute position of the first row of this pass = sequence length before it
    int32_t seq;     // sequence index
    int32_t rows;    // rows in this pass (1 for decode)
};

struct SeqState {
    int32_t len;         // tokens in the cache
    int32_t next_token;  // greedy argmax of the current logits
};

// Geometry of the model and of the K/V cache, passed by value to kernels.
struct Geom {
    int32_t d, Hq, Hkv, dh, F, V;
    int32_t max_pos;
    float eps;
    float scale;            // 1/sqrt(dh)
    // K/V cache, element strides: [seq][layer][K | V | V^T][hi | lo][Hkv][max_pos][dh].  The lo plane
    // exists only in the paired bf16 format, where a value is stored as bf16(x) + bf16(x - bf16(x)).
    // V^T (same size per head, laid out by vt_tile_off) exists only with the append-chunk path: its PV product
    // on the matrix cores needs 8 consecutive positions of one channel in one register quad.
    // max_pos is the allocated row count (capacity rounded up to a multiple of 32).
    size_t kv_head_stride, kv_v_offset, kv_lo_offset /* 0: no lo plane */, kv_vt_offset /* 0: no V^T */;
    size_t kv_layer_stride, kv_seq_stride;
};

// Offset (elements, relative to the head's plane) of value (pos, channel) in the transposed V planes (head_dim 128).
// Per tile of 32 positions the 128 x 32 block is stored in matrix-core A-operand order of the P V product:
// [tile][channel / 32][position bit 3][position bit 4][channel % 32][position % 8], so the 64 lanes of a wave read
// one contiguous KiB per instruction.
__host__ __device__ inline size_t vt_tile_off(int pos, int ch) {
    return ((((size_t)(pos >> 5) * 4 + (ch >> 5)) * 2 + ((pos >> 3) & 1)) * 64 + ((pos >> 4) & 1) * 32 + (ch & 31)) * 8 + (pos & 7);
}

enum KernelClass {
    KC_BEGIN = 0, KC_EMBED, KC_QKV, KC_ATTN, KC_OPROJ, KC_GATEUP, KC_DOWN, KC_LMHEAD, KC_ARGMAX,
    KC_CHUNK_PREP, KC_CHUNK_GEMM, KC_CHUNK_ATTN, KC_CHUNK_MISC,
    // phases inside the fused decoding kernel (time stamps of workgroup 0): work, then wait at the grid barrier
    KC_F_TOTAL, KC_F_QKV, KC_F_QKV_WAIT, KC_F_ATTN, KC_F_ATTN_WAIT, KC_F_MERGE, KC_F_MERGE_WAIT, KC_F_OPROJ, KC_F_OPROJ_WAIT,
    KC_F_GATEUP, KC_F_GATEUP_WAIT, KC_F_DOWN, KC_F_DOWN_WAIT, KC_F_HEAD, KC_F_HEAD_WAIT, KC_COUNT
};

// ---- device helpers -------------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (inputs are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPL = 4;   // elements in one 16-byte lane load
    __device__ static __forceinline__ void expand(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static __forceinline__ float load1(const float* p) { return *p; }
    __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int EPL = 8;
    __device__ static __forceinline__ void expand(const uint4& v, float (&f)[8]) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
    __device__ static __forceinline__ float load1(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
    __device__ static __forceinline__ void store1(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16-byte loads through pointers that are known to be global memory (a pointer read from a table in
// memory is otherwise treated as generic and loaded with flat instructions, which also count as LDS
// traffic when the wave waits for its LDS reads).
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;
typedef const __attribute__((address_space(1))) float* global_f32_ptr;

// streaming variant: data that is read once (weights)
__device__ __forceinline__ uint4 load16_stream(const void* p) {
    u32x4 v = __builtin_nontemporal_load((global_u32x4_ptr)(uintptr_t)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load16(const void* p) {
    u32x4 v = *(global_u32x4_ptr)(uintptr_t)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float load_f32(const float* p) { return *(global_f32_ptr)(uintptr_t)p; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace asynclm
