// Batch-1 decoding step on gfx950: bandwidth-bound matrix-vector kernels with fused
// RMSNorm / rotary / K-V write / SwiGLU / residual epilogues, split-sequence attention,
// on-device greedy argmax.  All activations stay in fp32; only weights and K/V are stored
// in the model's dtype.
#include "common.h"
#include "launch.h"
#include "decode_device.h"

#include <algorithm>

namespace asynclm {

// ---------------------------------------------------------------------------------------------
// step bookkeeping
// ---------------------------------------------------------------------------------------------

// Chooses the token of this step (forced, or the greedy one left by the previous forward pass),
// publishes it and its position to the step descriptor, and grows the sequence by one.
// token_early: optional host-visible word that also receives the token, so that the host can read it as soon as this
// kernel has run instead of after the whole step.
// pipe_abort: the give-up word of a step that runs on two streams, cleared here (this kernel runs alone, after the
// previous step has ended and before any kernel of this one starts); the step number goes up by one.
__global__ void k_begin_step(StepDesc* step, SeqState* st, int32_t seq, int32_t forced, int32_t* token_log, int32_t* token_early,
                             unsigned* pipe_abort) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (pipe_abort) *pipe_abort = 0u;
        step->epoch = (step->epoch + 1) & 0x3fffff;
        SeqState s = st[seq];
        int32_t tok = forced >= 0 ? forced : s.next_token;
        step->token = tok;
        step->pos = s.len;
        step->seq = seq;
        step->rows = 1;
        st[seq].len = s.len + 1;
        *token_log = tok;
        if (token_early) *token_early = tok;
    }
}

template <typename WT>
__global__ __launch_bounds__(256) void k_embed(const WT* __restrict__ E, const StepDesc* __restrict__ step,
                                               float* __restrict__ x, int d) {
    const WT* row = E + (size_t)step->token * d;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d; i += gridDim.x * 256) x[i] = Elem<WT>::load1(row + i);
}

// ---------------------------------------------------------------------------------------------
// matrix-vector product, one row pair ("unit") per wave at a time
// ---------------------------------------------------------------------------------------------

struct GemvArgs {
    const void* W;          // [rows, K] row-major
    int32_t rows, K;
    int32_t units;          // row pairs to compute
    int32_t uq, ur;         // units / waves of the grid, units % waves (set by the launcher)
    int32_t done_cap;       // finished row pairs a wave can park in LDS
    const float* x;         // [K] fp32 input vector
    const float* gain;      // [K] RMSNorm gain, or nullptr for no normalisation
    float* y;               // output (meaning depends on the epilogue)
    const float* res;       // residual input (EPI_RESID)
    float* q_out;           // EPI_QKV: rotated queries [Hq*dh]
    void* kv_layer;         // EPI_QKV: this layer's K plane of sequence 0
    const float* rope_cos;  // [max_pos, dh/2]
    const float* rope_sin;
    const StepDesc* step;
    int32_t layer;
    int32_t y_seq_stride;   // EPI_STORE: y is the row step->seq of a [sequences][y_seq_stride] array
    // merged attention output as input vector (x == nullptr): see VecSource
    const float* part_acc; const float* part_ml; int32_t merge_nsplit, merge_dh, merge_hq;
    PipeSync sync;          // hand-over from / to the neighbouring kernels of a step that runs on two streams
};

// Every wave owns a contiguous share of the row pairs and streams them through a ring of four register
// tiles (decode_device.h); the first tiles are requested before the input vector is staged.
// PIPE: the kernel may start while the kernel that produces its input vector is still running (two streams).  It then
// requests its first weight tiles, waits for the producer's workgroups (PipeSync), and only then reads the vector;
// its own results are written through, and when they have arrived it counts itself into its own flag.  Two workgroups of such kernels
// fit one compute unit (launch bounds), so the workgroups of two neighbouring kernels are always all resident.
// MODE 0: the default kernel; 1 (PIPE): the two-stream variant above; 2 (STAMP): the default kernel leaving time stamps
// (stamp mode of the one-stream step).  The stamps are a variant of their own because even a skipped clock read at the
// start of the kernel costs a microsecond: the branch around it waits for one kernel argument before the other argument
// loads are issued.
template <typename WT, int EPI, int NB, int MODE>
__global__ __launch_bounds__(256, MODE == 1 ? 2 : 1) void k_gemv(GemvArgs a, Geom g) {
    constexpr bool PIPE = MODE == 1, STAMP = MODE == 2;
    constexpr int EPL = Elem<WT>::EPL;
    extern __shared__ float4 lds4[];
    __shared__ float red[4];
    __shared__ int s_go;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (PIPE) pipe_stamp(a.sync, 0);
    const unsigned long long t_start = STAMP ? wall_clock64() : 0ull;      // stored at the kernel's end

    // NB > 0 (the vector is a plain one that fits one batch of NB x 16 bytes per thread; with a gain in the
    // normalising products, without in the residual ones): it is requested before the first weight tiles, so it is
    // back and staged long before them, and the first tile is multiplied as soon as it arrives.  NB = 0: the vector
    // (any source) is staged after the requests.
    constexpr int NB1 = NB > 0 ? NB : 1;
    constexpr bool GAIN = EPI != EPI_RESID;
    EarlyBatch<NB1, GAIN> vb;
    if (NB > 0 && !PIPE) {
        early_request(vb, a.x, a.gain, a.K);
        __builtin_amdgcn_sched_barrier(0);
    }
    Phase<WT> ph = make_phase_split<WT, EPI>(a.W, a.rows, a.K, a.units, a.uq, a.ur);
    const int plane_stride = ph.KT * 256 + 64;
    float4* done = lds4 + (size_t)plane_stride * (EPL / 4) + (size_t)wave * a.done_cap;
    Slot ring[RING];
    Cursor lc;
    phase_prefetch_w<WT, EPI>(ring, ph, lane, g);
    EpiOut eo;
    eo.y = a.y; eo.res = a.res; eo.q_out = a.q_out; eo.kv_layer = a.kv_layer;
    eo.rope_cos = a.rope_cos; eo.rope_sin = a.rope_sin; eo.rows = a.rows; eo.pos = 0; eo.seq = 0;
    if (EPI == EPI_QKV) { eo.pos = a.step->pos; eo.seq = a.step->seq; }
    if (EPI == EPI_STORE) eo.y += (size_t)a.step->seq * a.y_seq_stride;      // the logits row of the step's sequence
    if (PIPE) {
        // nothing but weights before the hand-over: the residual may come from the kernel before the previous one,
        // which is only known to be complete once the previous one is
        __builtin_amdgcn_sched_barrier(0);
        if (!pipe_wait(a.sync, &s_go)) return;
        if (NB > 0) early_request(vb, a.x, a.gain, a.K);
        __builtin_amdgcn_sched_barrier(0);
    }
    phase_prefetch_e<WT, EPI>(ring, ph, lc, g, eo);

    float ssq;
    if (NB > 0) ssq = early_stage<WT, NB1, GAIN>(vb, lds4, plane_stride, a.K, ph.Kg, ph.KT, red);
    else {
        VecSource vs{a.x, a.gain, a.part_acc, a.part_ml, a.merge_nsplit, a.merge_dh, a.merge_hq};
        ssq = stage_vector<WT, (EPI == EPI_RESID ? 16 : 4)>(lds4, plane_stride, vs, a.K, ph.Kg, ph.KT, true, red);
    }
    const float nscale = a.gain ? rsqrtf(ssq / (float)a.K + g.eps) : 1.f;
    const unsigned long long t_staged = STAMP ? wall_clock64() : 0ull;
    float best_v = -INFINITY; int best_i = 0x7fffffff;
    phase_run<WT, EPI>(ring, ph, lc, lds4, plane_stride, nscale, eo, g, lane, done, best_v, best_i);
    if (PIPE) pipe_signal(a.sync, &s_go);
    if (STAMP) step_stamp_done(a.sync, t_start, t_staged);
}

// The finishing-time words of every workgroup of every kernel of a step in stamp mode start at zero.
__global__ void k_stamp_init(unsigned long long* done_wg, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) done_wg[i] = 0ull;
}

hipError_t launch_stamp_init(unsigned long long* done_wg, int kernels, hipStream_t s) {
    hipLaunchKernelGGL(k_stamp_init, dim3(64), dim3(256), 0, s, done_wg, (size_t)kernels * STAMP_DONE_SLOTS);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// split-sequence decode attention: one query per head against the cached prefix
// ---------------------------------------------------------------------------------------------

struct AttnArgs {
    const float* q;         // [Hq*dh], rotated, unscaled
    const void* kv_layer;   // this layer's K plane of sequence 0
    const StepDesc* step;
    float* o;               // [Hq*dh]
    float* part_acc;        // [Hq][nsplit][dh]
    float* part_ml;         // [Hq][nsplit][2]
    int32_t* counters;      // [Hkv], zero between launches
    int32_t nsplit;
    int32_t defer_merge;    // 1: leave the partials to the O projection (no merge here, even for one split)
    PipeSync sync;
};

// PIPE: see k_gemv.  The query and the newest cache row come from the QKV kernel of the same step, which may still be
// running when this kernel starts: neither the query nor any cache row is read before its hand-over.
template <typename KVT, int DH, int G, bool PAIR, bool PIPE>
__global__ __launch_bounds__(256, PIPE ? 2 : 1) void k_attn_decode(AttnArgs a, Geom g) {
    constexpr int EPL = Elem<KVT>::EPL;
    constexpr int PPW = 64 / (DH / EPL);        // positions per wave-wide load
    extern __shared__ float lds[];
    __shared__ int s_last;
    __shared__ int s_go;

    const int tid = threadIdx.x;
    const int kvh = blockIdx.x, split = blockIdx.y, nsplit = a.nsplit;
    const int len = a.step->pos + 1;
    if (PIPE) pipe_stamp(a.sync, 0);
    if (PIPE && !pipe_wait(a.sync, &s_go)) return;
    // split boundaries: equal shares rounded up to whole workgroup rounds
    const int quantum = 4 * PPW;
    int per = (len + nsplit - 1) / nsplit;
    per = (per + quantum - 1) / quantum * quantum;
    const int s0 = min(split * per, len), s1 = min(s0 + per, len);

    const KVT* Kp = (const KVT*)a.kv_layer + (size_t)a.step->seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
    const KVT* Vp = Kp + g.kv_v_offset;
    float mh[G], lh[G];
    attn_split<KVT, DH, G, PAIR>(a.q, Kp, Vp, g.kv_lo_offset, kvh, s0, s1, g.scale, lds, mh, lh);

    for (int t = tid; t < G * DH; t += 256) {
        const int h = t / DH, dim = t - h * DH;
        const float A = attn_gather<KVT, DH, G>(lds, h, dim);
        float M = mh[0], L = lh[0];
#pragma unroll
        for (int hh = 1; hh < G; ++hh) if (hh == h) { M = mh[hh]; L = lh[hh]; }
        const int hq = kvh * G + h;
        if (nsplit == 1 && !a.defer_merge) {
            store_coherent(a.o + hq * DH + dim, A / L);
        } else {
            store_coherent(a.part_acc + ((size_t)hq * nsplit + split) * DH + dim, A);
            if (dim == 0) {
                store_coherent(a.part_ml + ((size_t)hq * nsplit + split) * 2, M);
                store_coherent(a.part_ml + ((size_t)hq * nsplit + split) * 2 + 1, L);
            }
        }
    }
    if (nsplit == 1 || a.defer_merge) {
        if (PIPE) pipe_signal(a.sync, &s_go);
        return;
    }

    // the workgroup that finishes last for this kv head merges the splits, in split order
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = atomicAdd(&a.counters[kvh], 1);
        s_last = (ticket == nsplit - 1);
    }
    __syncthreads();
    if (!s_last) {
        if (PIPE) pipe_signal(a.sync, &s_go);
        return;
    }
    __threadfence();
    // weights of the splits: f_s = exp(m_s - M) / L, one wave per head at a time, lane = split
    __syncthreads();                              // the partial accumulators in LDS have been read
    float* s_f = lds;                             // [G][ATTN_MAX_SPLIT] factors
    {
        const int lane = tid & 63, wave = tid >> 6;
        for (int h = wave; h < G; h += 4) {
            const float* ml = a.part_ml + (size_t)(kvh * G + h) * nsplit * 2;
            const float ms = lane < nsplit ? ml[lane * 2] : -INFINITY;
            const float ls = lane < nsplit ? ml[lane * 2 + 1] : 0.f;
            const float M = wave_max_all(ms);
            const float f = ms > -INFINITY ? expf(ms - M) : 0.f;
            const float L = wave_sum_all(ls * f);
            s_f[h * ATTN_MAX_SPLIT + lane] = f / L;
        }
    }
    __syncthreads();
    // thread = (output float4, half of the splits); the two halves meet in LDS
    {
        constexpr int NO = G * DH / 4;            // output float4s of this kv head
        float4* s_half = reinterpret_cast<float4*>(lds + G * ATTN_MAX_SPLIT);
        for (int base = 0; base < NO; base += 128) {
            const int t = base + (tid & 127), half = tid >> 7;
            const int tc = min(t, NO - 1);
            const int h = tc / (DH / 4), d4 = tc - h * (DH / 4), hq = kvh * G + h;
            const float4* src = (const float4*)(a.part_acc + (size_t)hq * nsplit * DH) + d4;
            const int per = (nsplit + 1) / 2, sp0 = half * per, sp1 = min(nsplit, sp0 + per);
            float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int sp = sp0; sp < sp1; sp += 8) {
                float4 v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = src[(size_t)min(sp + k, sp1 - 1) * (DH / 4)];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float f = sp + k < sp1 ? s_f[h * ATTN_MAX_SPLIT + min(sp + k, ATTN_MAX_SPLIT - 1)] : 0.f;
                    r.x = fmaf(v[k].x, f, r.x); r.y = fmaf(v[k].y, f, r.y); r.z = fmaf(v[k].z, f, r.z); r.w = fmaf(v[k].w, f, r.w);
                }
            }
            if (half == 1) s_half[tid & 127] = r;
            __syncthreads();
            if (half == 0 && t < NO) {
                const float4 o2 = s_half[tid];
                float* op = a.o + (size_t)hq * DH + 4 * d4;
                store_coherent(op, r.x + o2.x); store_coherent(op + 1, r.y + o2.y);
                store_coherent(op + 2, r.z + o2.z); store_coherent(op + 3, r.w + o2.w);
            }
            __syncthreads();
        }
    }
    if (tid == 0) a.counters[kvh] = 0;
    if (PIPE) pipe_signal(a.sync, &s_go);
}

// ---------------------------------------------------------------------------------------------
// greedy argmax over the vocabulary: per-block (max, lowest index), last block merges
// ---------------------------------------------------------------------------------------------

// (max, lowest index) over logits[0..V) without the `nban` ids in `ban`: per-block results in part_v / part_i, the block
// that arrives last (counter, zero between launches) merges them and stores the index to *out.
__device__ __forceinline__ void argmax_blocks(const float* __restrict__ logits, int V, const int32_t* __restrict__ ban, int nban,
                                              float* part_v, int32_t* part_i, int32_t* counter, int32_t* out) {
    __shared__ float sv[4];
    __shared__ int si[4];
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nb = gridDim.x;
    const int per = (V + nb - 1) / nb;
    const int i0 = blockIdx.x * per, i1 = min(V, i0 + per);
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int i = i0 + tid; i < i1; i += 256) {
        bool allowed = true;
        for (int k = 0; k < nban; ++k) allowed = allowed && i != ban[k];
        if (allowed) amax_merge(bv, bi, logits[i], i);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
        amax_merge(bv, bi, ov, oi);
    }
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) amax_merge(bv, bi, sv[w], si[w]);
        part_v[blockIdx.x] = bv; part_i[blockIdx.x] = bi;
        __threadfence();
        s_last = (atomicAdd(counter, 1) == nb - 1);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    bv = -INFINITY; bi = 0x7fffffff;
    for (int b = tid; b < nb; b += 256) amax_merge(bv, bi, __builtin_nontemporal_load(part_v + b), __builtin_nontemporal_load(part_i + b));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
        amax_merge(bv, bi, ov, oi);
    }
    __syncthreads();
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) amax_merge(bv, bi, sv[w], si[w]);
        *out = bi;
        *counter = 0;
    }
}

__global__ __launch_bounds__(256) void k_argmax(const float* __restrict__ logits_base, int V, const StepDesc* step,
                                                SeqState* st, float* part_v, int32_t* part_i, int32_t* counter,
                                                const int32_t* __restrict__ banned, int seq_arg) {
    const int seq = seq_arg >= 0 ? seq_arg : step->seq;
    const int32_t* ban = banned + (size_t)seq * (1 + BAN_MAX);
    argmax_blocks(logits_base + (size_t)seq * V, V, ban + 1, ban[0], part_v, part_i, counter, &st[seq].next_token);
}

// The same choice for a caller that brings the logits, the ids to skip and the place for the result itself.
__global__ __launch_bounds__(256) void k_argmax_flat(const float* __restrict__ logits, int V, const int32_t* __restrict__ ban, int nban,
                                                     float* part_v, int32_t* part_i, int32_t* counter, int32_t* out) {
    argmax_blocks(logits, V, ban, nban, part_v, part_i, counter, out);
}

__global__ void k_clear_word(int32_t* p) { *p = 0; }

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

static int g_gemv_grid = 256;       // workgroups per matrix-vector kernel; decode_init sets it to the number of compute units
static size_t g_gemv_lds_limit = 48 * 1024;   // dynamic LDS a matrix-vector kernel may ask for (raised by decode_init)

// Early request of the vector when it is a plain one that fits one batch: 4 or 8 x 16 bytes per thread (with as
// many of the gain) in the normalising products, 4 or 16 in the residual ones.
template <int EPI> struct EarlyNB { static constexpr int SMALL = 4, LARGE = EPI == EPI_RESID ? 16 : 8, HUGE = 32; };

template <typename WT, int EPI, int NB>
static const void* gemv_func_n(int mode) {
    return mode == 1 ? (const void*)(k_gemv<WT, EPI, NB, 1>) : mode == 2 ? (const void*)(k_gemv<WT, EPI, NB, 2>) : (const void*)(k_gemv<WT, EPI, NB, 0>);
}

// The instantiation that serves a product with K columns (plain_x: the input is a plain vector, not split partials).
template <typename WT, int EPI>
static const void* gemv_func(int K, bool plain_x, int pipe /* mode: 0 default, 1 two-stream, 2 stamps */) {
    if (plain_x && K <= 1024 * EarlyNB<EPI>::SMALL) return gemv_func_n<WT, EPI, EarlyNB<EPI>::SMALL>(pipe);
    if (plain_x && K <= 1024 * EarlyNB<EPI>::LARGE) return gemv_func_n<WT, EPI, EarlyNB<EPI>::LARGE>(pipe);
    if (EPI == EPI_RESID && plain_x && K <= 1024 * EarlyNB<EPI>::HUGE) return gemv_func_n<WT, EPI_RESID, EarlyNB<EPI_RESID>::HUGE>(pipe);
    return gemv_func_n<WT, EPI, 0>(pipe);
}

template <typename WT>
static size_t gemv_lds_bytes(int K, int units, int grid, int* done_cap) {
    *done_cap = (units + grid * 4 - 1) / (grid * 4) + 1;
    const int kg = K / Elem<WT>::EPL, kt = (kg + 255) / 256;
    return (size_t)(kt * 256 + 64) * Elem<WT>::EPL * sizeof(float) + (size_t)4 * (*done_cap) * sizeof(float4);
}

template <typename WT, int EPI>
static hipError_t launch_gemv_t(const GemvArgs& a0, const Geom& g, hipStream_t s) {
    GemvArgs a = a0;
    const size_t lds = gemv_lds_bytes<WT>(a.K, a.units, g_gemv_grid, &a.done_cap);
    a.uq = a.units / (g_gemv_grid * 4); a.ur = a.units % (g_gemv_grid * 4);
    if (lds > g_gemv_lds_limit) return hipErrorInvalidValue;
    if (EPI != EPI_RESID && !(a.x && a.gain)) return hipErrorInvalidValue;   // the normalising products take a vector and a gain
    if (EPI == EPI_RESID && a.gain) return hipErrorInvalidValue;
    const int mode = (a.sync.go_wait || a.sync.go_signal) ? 1 : a.sync.done_wg ? 2 : 0;
    Geom gg = g;
    void* params[] = {&a, &gg};
    return hipLaunchKernel(gemv_func<WT, EPI>(a.K, a.x != nullptr, mode), dim3(g_gemv_grid), dim3(256), params, lds, s);
}

template <typename WT>
static hipError_t launch_gemv_w(int epi, const GemvArgs& a, const Geom& g, hipStream_t s) {
    switch (epi) {
        case EPI_STORE: return launch_gemv_t<WT, EPI_STORE>(a, g, s);
        case EPI_RESID: return launch_gemv_t<WT, EPI_RESID>(a, g, s);
        case EPI_SWIGLU: return launch_gemv_t<WT, EPI_SWIGLU>(a, g, s);
        default: return launch_gemv_t<WT, EPI_QKV>(a, g, s);
    }
}

template <typename WT, int EPI, int PIPE /* mode */>
static hipError_t set_lds_p(int bytes) {
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, 0, PIPE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, EarlyNB<EPI>::SMALL, PIPE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, EarlyNB<EPI>::LARGE, PIPE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if (EPI != EPI_RESID) return hipSuccess;
    return hipFuncSetAttribute((const void*)(k_gemv<WT, EPI_RESID, EarlyNB<EPI_RESID>::HUGE, PIPE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}
template <typename WT, int EPI>
static hipError_t set_lds_t(int bytes) {
    hipError_t e = set_lds_p<WT, EPI, 0>(bytes);
    if (!e) e = set_lds_p<WT, EPI, 1>(bytes);
    return e ? e : set_lds_p<WT, EPI, 2>(bytes);
}

void decode_set_gemv_grid(int grid) { g_gemv_grid = grid; }

hipError_t decode_init(int dtype, int max_k) {
    {   // one workgroup per compute unit measured best: every workgroup stages the whole input vector
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            g_gemv_grid = cus;
    }
    // staged vector with its padding + parked units (16 KiB cover 256 units per wave), within the 160 KiB of a compute unit
    const int bytes = std::min((max_k + 8 * 256 + 64 * 8) * (int)sizeof(float) + 16 * 1024, 160 * 1024);
    // process-wide, shared by every context: only ever raised
    if ((size_t)bytes <= g_gemv_lds_limit) return hipSuccess;
    hipError_t e;
    if (dtype == 0) {
        if ((e = set_lds_t<float, EPI_STORE>(bytes))) return e;
        if ((e = set_lds_t<float, EPI_RESID>(bytes))) return e;
        if ((e = set_lds_t<float, EPI_SWIGLU>(bytes))) return e;
        if ((e = set_lds_t<float, EPI_QKV>(bytes))) return e;
    } else {
        if ((e = set_lds_t<bf16_t, EPI_STORE>(bytes))) return e;
        if ((e = set_lds_t<bf16_t, EPI_RESID>(bytes))) return e;
        if ((e = set_lds_t<bf16_t, EPI_SWIGLU>(bytes))) return e;
        if ((e = set_lds_t<bf16_t, EPI_QKV>(bytes))) return e;
    }
    g_gemv_lds_limit = (size_t)bytes;
    return hipSuccess;
}

static hipError_t launch_gemv(int dtype, int epi, const GemvArgs& a, const Geom& g, hipStream_t s) {
    return dtype == 0 ? launch_gemv_w<float>(epi, a, g, s) : launch_gemv_w<bf16_t>(epi, a, g, s);
}

hipError_t launch_begin_step(const DecodeBuffers& b, int seq, int forced, int32_t* token_early, hipStream_t s) {
    hipLaunchKernelGGL(k_begin_step, dim3(1), dim3(64), 0, s, b.step, b.seq_state, seq, forced, b.token_log, token_early, b.pipe_abort);
    return hipGetLastError();
}

int decode_gemv_grid() { return g_gemv_grid; }

hipError_t launch_embed(int dtype, const void* E, const DecodeBuffers& b, const Geom& g, hipStream_t s) {
    const int grid = (g.d + 255) / 256;
    if (dtype == 0) hipLaunchKernelGGL(k_embed<float>, dim3(grid), dim3(256), 0, s, (const float*)E, b.step, b.x, g.d);
    else hipLaunchKernelGGL(k_embed<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)E, b.step, b.x, g.d);
    return hipGetLastError();
}

hipError_t launch_qkv(int dtype, const void* wqkv, const float* gain, void* kv_layer, const DecodeBuffers& b,
                      const Geom& g, hipStream_t s, const PipeSync* sync) {
    GemvArgs a{};
    if (sync) a.sync = *sync;
    a.W = wqkv; a.rows = (g.Hq + 2 * g.Hkv) * g.dh; a.K = g.d; a.units = a.rows / 2;
    a.x = b.x; a.gain = gain; a.q_out = b.q; a.kv_layer = kv_layer;
    a.rope_cos = b.rope_cos; a.rope_sin = b.rope_sin; a.step = b.step;
    return launch_gemv(dtype, EPI_QKV, a, g, s);
}

hipError_t launch_oproj(int dtype, const void* wo, int merge_nsplit, const DecodeBuffers& b, const Geom& g, hipStream_t s,
                        const PipeSync* sync, float* x_out) {
    GemvArgs a{};
    if (sync) a.sync = *sync;
    a.W = wo; a.rows = g.d; a.K = g.Hq * g.dh; a.units = (a.rows + 1) / 2;
    a.x = b.o; a.gain = nullptr; a.y = x_out ? x_out : b.x; a.res = b.x; a.step = b.step;
    if (merge_nsplit > 0) {
        if (merge_nsplit > MERGE_MAX_SPLIT) return hipErrorInvalidValue;
        a.x = nullptr; a.part_acc = b.part_acc; a.part_ml = b.part_ml;
        a.merge_nsplit = merge_nsplit; a.merge_dh = g.dh; a.merge_hq = g.Hq;
    }
    return launch_gemv(dtype, EPI_RESID, a, g, s);
}

hipError_t launch_gateup(int dtype, const void* wgu, const float* gain, const DecodeBuffers& b, const Geom& g, hipStream_t s,
                         const PipeSync* sync, const float* x_in) {
    GemvArgs a{};
    if (sync) a.sync = *sync;
    a.W = wgu; a.rows = 2 * g.F; a.K = g.d; a.units = g.F;
    a.x = x_in ? x_in : b.x; a.gain = gain; a.y = b.a; a.step = b.step;
    return launch_gemv(dtype, EPI_SWIGLU, a, g, s);
}

hipError_t launch_down(int dtype, const void* wd, const DecodeBuffers& b, const Geom& g, hipStream_t s, const PipeSync* sync,
                       const float* res_in) {
    GemvArgs a{};
    if (sync) a.sync = *sync;
    a.W = wd; a.rows = g.d; a.K = g.F; a.units = (a.rows + 1) / 2;
    a.x = b.a; a.gain = nullptr; a.y = b.x; a.res = res_in ? res_in : b.x; a.step = b.step;
    return launch_gemv(dtype, EPI_RESID, a, g, s);
}

hipError_t launch_lmhead(int dtype, const void* wout, const float* gain, float* logits_base, const DecodeBuffers& b,
                         const Geom& g, hipStream_t s, const PipeSync* sync) {
    GemvArgs a{};
    if (sync) a.sync = *sync;
    a.W = wout; a.rows = g.V; a.K = g.d; a.units = (a.rows + 1) / 2;
    a.x = b.x; a.gain = gain; a.y = logits_base; a.y_seq_stride = g.V; a.step = b.step;
    return launch_gemv(dtype, EPI_STORE, a, g, s);
}

template <typename KVT, int DH, bool PAIR>
static hipError_t launch_attn_t(const AttnArgs& a, const Geom& g, hipStream_t s) {
    const dim3 grid(g.Hkv, a.nsplit), block(256);
    const bool pipe = a.sync.go_wait || a.sync.go_signal;
#define ATTN_CASE(GG)                                                                                                   \
    case GG: {                                                                                                          \
        const size_t lds = sizeof(float) * attn_lds_floats<KVT, DH, GG>();                                              \
        if (lds > 48 * 1024) {                                                                                          \
            hipError_t e = hipFuncSetAttribute(pipe ? (const void*)(k_attn_decode<KVT, DH, GG, PAIR, true>)             \
                                                    : (const void*)(k_attn_decode<KVT, DH, GG, PAIR, false>),           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                   \
            if (e) return e;                                                                                            \
        }                                                                                                               \
        if (pipe) hipLaunchKernelGGL((k_attn_decode<KVT, DH, GG, PAIR, true>), grid, block, lds, s, a, g);              \
        else hipLaunchKernelGGL((k_attn_decode<KVT, DH, GG, PAIR, false>), grid, block, lds, s, a, g);                  \
        break;                                                                                                          \
    }
    switch (g.Hq / g.Hkv) {
        ATTN_CASE(1) ATTN_CASE(2) ATTN_CASE(4) ATTN_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef ATTN_CASE
    return hipGetLastError();
}

hipError_t launch_attn_decode(int dtype, const void* kv_layer, int nsplit, bool merge_in_oproj, const DecodeBuffers& b,
                              const Geom& g, hipStream_t s, const PipeSync* sync) {
    AttnArgs a{};
    if (sync) a.sync = *sync;
    a.defer_merge = merge_in_oproj ? 1 : 0;
    a.q = b.q; a.kv_layer = kv_layer; a.step = b.step; a.o = b.o;
    a.part_acc = b.part_acc; a.part_ml = b.part_ml; a.counters = b.attn_counters; a.nsplit = nsplit;
    if (dtype == 0) return g.dh == 64 ? launch_attn_t<float, 64, false>(a, g, s) : launch_attn_t<float, 128, false>(a, g, s);
    if (g.kv_lo_offset) return g.dh == 64 ? launch_attn_t<bf16_t, 64, true>(a, g, s) : launch_attn_t<bf16_t, 128, true>(a, g, s);
    return g.dh == 64 ? launch_attn_t<bf16_t, 64, false>(a, g, s) : launch_attn_t<bf16_t, 128, false>(a, g, s);
}

hipError_t launch_argmax_flat(const float* logits, int n, const int32_t* ban, int nban, float* part_v, int32_t* part_i,
                              int32_t* counter, int32_t* out, hipStream_t s) {
    int nb = (n + 2047) / 2048;
    if (nb > ARGMAX_MAX_BLOCKS) nb = ARGMAX_MAX_BLOCKS;
    hipLaunchKernelGGL(k_clear_word, dim3(1), dim3(1), 0, s, counter);      // whatever an earlier launch left there
    hipLaunchKernelGGL(k_argmax_flat, dim3(nb), dim3(256), 0, s, logits, n, ban, nban, part_v, part_i, counter, out);
    return hipGetLastError();
}

hipError_t launch_argmax(const float* logits_base, const DecodeBuffers& b, const Geom& g, hipStream_t s, int seq) {
    int nb = (g.V + 2047) / 2048;
    if (nb > ARGMAX_MAX_BLOCKS) nb = ARGMAX_MAX_BLOCKS;
    hipLaunchKernelGGL(k_argmax, dim3(nb), dim3(256), 0, s, logits_base, g.V, b.step, b.seq_state, b.amax_v, b.amax_i, b.amax_counter, b.banned, seq);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// two-stream step: can the workgroups of two neighbouring kernels always all be resident?
// ---------------------------------------------------------------------------------------------

template <typename KVT, int DH, bool PAIR>
static const void* attn_func_pipe(int G, size_t* lds) {
    switch (G) {
        case 1: *lds = sizeof(float) * attn_lds_floats<KVT, DH, 1>(); return (const void*)(k_attn_decode<KVT, DH, 1, PAIR, true>);
        case 2: *lds = sizeof(float) * attn_lds_floats<KVT, DH, 2>(); return (const void*)(k_attn_decode<KVT, DH, 2, PAIR, true>);
        case 4: *lds = sizeof(float) * attn_lds_floats<KVT, DH, 4>(); return (const void*)(k_attn_decode<KVT, DH, 4, PAIR, true>);
        case 8: *lds = sizeof(float) * attn_lds_floats<KVT, DH, 8>(); return (const void*)(k_attn_decode<KVT, DH, 8, PAIR, true>);
        default: return nullptr;
    }
}

template <typename WT>
static bool pipeline_fits_t(const Geom& g, bool kv_pair) {
    struct Item { const void* f; size_t lds; };
    Item items[6];
    int dc = 0, n = 0;
    const int nqkv = (g.Hq + 2 * g.Hkv) * g.dh, qd = g.Hq * g.dh, grid = g_gemv_grid;
    items[n++] = {gemv_func<WT, EPI_QKV>(g.d, true, 1), gemv_lds_bytes<WT>(g.d, nqkv / 2, grid, &dc)};
    items[n++] = {gemv_func<WT, EPI_RESID>(qd, false, 1), gemv_lds_bytes<WT>(qd, (g.d + 1) / 2, grid, &dc)};   // merges the key splits
    items[n++] = {gemv_func<WT, EPI_RESID>(qd, true, 1), gemv_lds_bytes<WT>(qd, (g.d + 1) / 2, grid, &dc)};
    items[n++] = {gemv_func<WT, EPI_SWIGLU>(g.d, true, 1), gemv_lds_bytes<WT>(g.d, g.F, grid, &dc)};
    items[n++] = {gemv_func<WT, EPI_RESID>(g.F, true, 1), gemv_lds_bytes<WT>(g.F, (g.d + 1) / 2, grid, &dc)};
    items[n++] = {gemv_func<WT, EPI_STORE>(g.d, true, 1), gemv_lds_bytes<WT>(g.d, (g.V + 1) / 2, grid, &dc)};
    for (int i = 0; i < n; ++i) {
        int per_cu = 0;
        if (items[i].lds > g_gemv_lds_limit) return false;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, items[i].f, 256, items[i].lds) != hipSuccess || per_cu < 2) return false;
    }
    size_t lds = 0;
    const void* af = g.dh == 64 ? (kv_pair ? attn_func_pipe<WT, 64, true>(g.Hq / g.Hkv, &lds) : attn_func_pipe<WT, 64, false>(g.Hq / g.Hkv, &lds))
                                : (kv_pair ? attn_func_pipe<WT, 128, true>(g.Hq / g.Hkv, &lds) : attn_func_pipe<WT, 128, false>(g.Hq / g.Hkv, &lds));
    if (!af) return false;
    if (lds > 48 * 1024 && hipFuncSetAttribute(af, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return false;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, af, 256, lds) != hipSuccess || per_cu < 2) return false;
    return true;
}

bool decode_pipeline_fits(int dtype, const Geom& g, bool kv_pair) {
    if (dtype == 0) return pipeline_fits_t<float>(g, false);
    return pipeline_fits_t<bf16_t>(g, kv_pair);
}

}  // namespace asynclm
