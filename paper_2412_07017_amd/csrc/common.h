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
    int32_t epoch;   // number of the decoding step (k_begin_step counts it up): part of the hand-over words of PipeSync
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
    // on the matrix cores needs 8 consecutive positions of one channel in one register quad.  Models of that path
    // keep the row-major V only on request (it serves the single-row attention kernel).
    // max_pos is the allocated row count (capacity rounded up to a multiple of 32).
    size_t kv_head_stride, kv_v_offset /* 0: no row-major V */, kv_lo_offset /* 0: no lo plane */, kv_vt_offset /* 0: no V^T */;
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

// Write-through stores.  The dies of the device have an L2 cache each; data that one running kernel hands to another
// (no kernel boundary in between) is stored with relaxed atomic stores at device scope, which go through to memory,
// and the reader only touches it after the hand-over (PipeSync), on lines that no cache of its die can hold.
__device__ __forceinline__ void store_coherent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void store_coherent(bf16_t* p, bf16_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Hand-over between two kernels that run at the same time on two streams.  The producer's workgroups count
// themselves into `counter` once their write-through stores have completed; the workgroup that arrives last resets the
// counter and writes the hand-over word (step number and producer kernel number) into one cache line PER CONSUMER
// WORKGROUP, and consumer workgroup w polls only line w: a word that every waiting workgroup polls would keep one
// memory channel busy with polls and slow the weight stream of the kernel that is still running, which visits every
// channel.  Every wait is bounded: after PIPE_SPIN_LIMIT polls, or once another workgroup has given up, the workgroup
// sets `abort` (and the host-visible error word) and leaves, so a launch always drains.
constexpr int PIPE_LINE_WORDS = 32;         // one hand-over word per 128 bytes
constexpr int PIPE_MAX_WORKGROUPS = 256;    // workgroups of a kernel that takes part (lines per region)
constexpr int PIPE_REGIONS = 4;             // kernel k signals region k % 4 (at most two kernels are in flight)
struct PipeSync {
    const unsigned* go_wait;    // region written by the previous kernel; nullptr: the inputs are complete at kernel start
    unsigned* go_signal;        // region this kernel writes when all its workgroups are done; nullptr: nobody waits
    unsigned* counter;          // arrivals of this kernel's workgroups (zero between kernels)
    unsigned* abort;            // shared by all kernels of a step
    int32_t* error_word;        // set to 1 when a wait gave up
    const StepDesc* step;       // step number
    unsigned wait_kernel, my_kernel;   // kernel numbers within the step
    unsigned long long* stamps; // optional, see pipe_stamp
    unsigned long long* done_wg; // optional, stamp mode of the one-stream step: see step_stamp_done
};
constexpr int STAMP_DONE_SLOTS = 1024;  // workgroups of a kernel whose finishing times are kept
constexpr unsigned PIPE_SPIN_LIMIT = 1u << 17;
#ifndef PIPE_POLL_SLEEP
#define PIPE_POLL_SLEEP 2      // x 64 clocks between two polls of a waiting workgroup
#endif

__device__ __forceinline__ unsigned pipe_word(const StepDesc* step, unsigned kernel) { return ((unsigned)step->epoch << 10) | kernel; }

// stamps[0..2]: start and hand-over seen of the first workgroup, done of the workgroup that finished first;
// stamps[3..5]: the same of the last workgroup / the workgroup that finished last.
__device__ __forceinline__ void pipe_stamp(const PipeSync& ps, int which) {
    if (!ps.stamps || threadIdx.x != 0) return;
    const bool first = blockIdx.x == 0 && blockIdx.y == 0, last = blockIdx.x == gridDim.x - 1 && blockIdx.y == gridDim.y - 1;
#ifdef PIPE_STAMP_ALL       // diagnosis builds: the latest start / hand-over seen over all workgroups
    if (first) ps.stamps[which] = wall_clock64();
    atomicMax(ps.stamps + 3 + which, (unsigned long long)wall_clock64());
#else
    if (first) ps.stamps[which] = wall_clock64();
    if (last) ps.stamps[3 + which] = wall_clock64();
#endif
}

// The 100 MHz clock if `on`, else 0.  The read takes about a microsecond and its result comes back with the kernel's
// argument loads, so it must not happen at all when no stamps are wanted; as an ordinary expression the compiler
// executes it anyway and selects (measured: 3.5 % of a decoding step), hence the volatile statement inside a branch.
__device__ __forceinline__ unsigned long long clock_if(bool on) {
    unsigned long long t = 0;
    if (on) asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t));
    return t;
}

// One-stream steps in stamp mode use words 0, 1, 3, 4 of the same six words per kernel (start and "input vector staged"
// of the first and of the last workgroup); every workgroup stores the time it is done to a word of its own (zero before
// the step), and the host takes the earliest and the latest (an atomic minimum / maximum on one word would cost 11 ns
// per workgroup, 3 us per kernel).  t_staged: the clock when the input vector was staged, read then and stored only
// here like the start: a store that may or may not happen among a kernel's requests would keep the compiler from
// counting the requests in flight, and it would wait for all of them (measured: 1.5-2 us per kernel).
// All threads of the workgroup call this.
__device__ __forceinline__ void step_stamp_done(const PipeSync& ps, unsigned long long t_start, unsigned long long t_staged) {
    if (!ps.done_wg) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const unsigned wg = blockIdx.y * gridDim.x + blockIdx.x;
    if (threadIdx.x == 0 && wg < (unsigned)STAMP_DONE_SLOTS) ps.done_wg[wg] = wall_clock64();
    if (threadIdx.x == 0 && ps.stamps) {
        if (wg == 0) { ps.stamps[0] = t_start; ps.stamps[1] = t_staged; }
        if (wg == gridDim.x * gridDim.y - 1) { ps.stamps[3] = t_start; ps.stamps[4] = t_staged; }
    }
}

// All threads of the workgroup call this; false: give up (uniform).
__device__ __forceinline__ bool pipe_wait(const PipeSync& ps, int* s_flag) {
    if (!ps.go_wait) { pipe_stamp(ps, 1); return true; }
    if (threadIdx.x == 0) {
        const unsigned want = pipe_word(ps.step, ps.wait_kernel);
        const unsigned* mine = ps.go_wait + (size_t)(blockIdx.y * gridDim.x + blockIdx.x) * PIPE_LINE_WORDS;
        int ok = 1;
        unsigned spins = 0;
        while (__hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != want) {
            __builtin_amdgcn_s_sleep(PIPE_POLL_SLEEP);
            ++spins;
            if (spins > PIPE_SPIN_LIMIT || ((spins & 255u) == 0 && __hip_atomic_load(ps.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) { ok = 0; break; }
        }
        if (!ok) {
            __hip_atomic_store(ps.abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *ps.error_word = 1;
        }
        *s_flag = ok;
    }
    pipe_stamp(ps, 1);
    __syncthreads();
    return *s_flag != 0;
}

// All threads call this after their last write-through store (256 threads per workgroup).
__device__ __forceinline__ void pipe_signal(const PipeSync& ps, int* s_flag) {
    if (!ps.go_signal) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this thread's write-through stores have completed
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned n = gridDim.x * gridDim.y;
        const unsigned ticket = __hip_atomic_fetch_add(ps.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (ps.stamps) {
            if (ticket == 0) ps.stamps[2] = wall_clock64();
            if (ticket == n - 1) ps.stamps[5] = wall_clock64();
        }
        if (ticket == n - 1) __hip_atomic_store(ps.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = ticket == n - 1;
    }
    __syncthreads();
    if (*s_flag) {
        const unsigned word = pipe_word(ps.step, ps.my_kernel);
        for (int w = threadIdx.x; w < PIPE_MAX_WORKGROUPS; w += blockDim.x)
            __hip_atomic_store(ps.go_signal + (size_t)w * PIPE_LINE_WORDS, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace asynclm
