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
__global__ void k_begin_step(StepDesc* step, SeqState* st, int32_t seq, int32_t forced, int32_t* token_log, int32_t* token_early) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
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
    // merged attention output as input vector (x == nullptr): see VecSource
    const float* part_acc; const float* part_ml; int32_t merge_nsplit, merge_dh, merge_hq;
};

// Every wave owns a contiguous share of the row pairs and streams them through a ring of four register
// tiles (decode_device.h); the first tiles are requested before the input vector is staged.
template <typename WT, int EPI, int NB>
__global__ __launch_bounds__(256) void k_gemv(GemvArgs a, Geom g) {
    constexpr int EPL = Elem<WT>::EPL;
    extern __shared__ float4 lds4[];
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    Phase<WT> ph = make_phase<WT, EPI>(a.W, a.rows, a.K, a.units);
    const int plane_stride = ph.KT * 256 + 64;
    float4* done = lds4 + (size_t)plane_stride * (EPL / 4) + (size_t)wave * a.done_cap;

    // NB > 0 (the vector is a plain one that fits one batch of NB x 16 bytes per thread; with a gain in the
    // normalising products, without in the residual ones): it is requested before the first weight tiles, so it is
    // back and staged long before them, and the first tile is multiplied as soon as it arrives.  NB = 0: the vector
    // (any source) is staged after the requests.
    constexpr int NB1 = NB > 0 ? NB : 1;
    constexpr bool GAIN = EPI != EPI_RESID;
    EarlyBatch<NB1, GAIN> vb;
    if (NB > 0) {
        early_request(vb, a.x, a.gain, a.K);
        __builtin_amdgcn_sched_barrier(0);
    }
    Slot ring[RING];
    Cursor lc;
    phase_prefetch_w<WT, EPI>(ring, ph, lane, g);
    EpiOut eo;
    eo.y = a.y; eo.res = a.res; eo.q_out = a.q_out; eo.kv_layer = a.kv_layer;
    eo.rope_cos = a.rope_cos; eo.rope_sin = a.rope_sin; eo.rows = a.rows; eo.pos = 0; eo.seq = 0;
    if (EPI == EPI_QKV) { eo.pos = a.step->pos; eo.seq = a.step->seq; }
    phase_prefetch_e<WT, EPI>(ring, ph, lc, g, eo);

    float ssq;
    if (NB > 0) ssq = early_stage<WT, NB1, GAIN>(vb, lds4, plane_stride, a.K, ph.Kg, ph.KT, red);
    else {
        VecSource vs{a.x, a.gain, a.part_acc, a.part_ml, a.merge_nsplit, a.merge_dh, a.merge_hq};
        ssq = stage_vector<WT, (EPI == EPI_RESID ? 16 : 4)>(lds4, plane_stride, vs, a.K, ph.Kg, ph.KT, true, red);
    }
    const float nscale = a.gain ? rsqrtf(ssq / (float)a.K + g.eps) : 1.f;
    float best_v = -INFINITY; int best_i = 0x7fffffff;
    phase_run<WT, EPI>(ring, ph, lc, lds4, plane_stride, nscale, eo, g, lane, done, best_v, best_i);
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
};

template <typename KVT, int DH, int G, bool PAIR>
__global__ __launch_bounds__(256) void k_attn_decode(AttnArgs a, Geom g) {
    constexpr int EPL = Elem<KVT>::EPL;
    constexpr int PPW = 64 / (DH / EPL);        // positions per wave-wide load
    extern __shared__ float lds[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int kvh = blockIdx.x, split = blockIdx.y, nsplit = a.nsplit;
    const int len = a.step->pos + 1;
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
            a.o[hq * DH + dim] = A / L;
        } else {
            a.part_acc[((size_t)hq * nsplit + split) * DH + dim] = A;
            if (dim == 0) { a.part_ml[((size_t)hq * nsplit + split) * 2] = M; a.part_ml[((size_t)hq * nsplit + split) * 2 + 1] = L; }
        }
    }
    if (nsplit == 1 || a.defer_merge) return;

    // the workgroup that finishes last for this kv head merges the splits, in split order
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = atomicAdd(&a.counters[kvh], 1);
        s_last = (ticket == nsplit - 1);
    }
    __syncthreads();
    if (!s_last) return;
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
                ((float4*)(a.o + (size_t)hq * DH))[d4] = make_float4(r.x + o2.x, r.y + o2.y, r.z + o2.z, r.w + o2.w);
            }
            __syncthreads();
        }
    }
    if (tid == 0) a.counters[kvh] = 0;
}

// ---------------------------------------------------------------------------------------------
// greedy argmax over the vocabulary: per-block (max, lowest index), last block merges
// ---------------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_argmax(const float* __restrict__ logits_base, int V, const StepDesc* step,
                                                SeqState* st, float* part_v, int32_t* part_i, int32_t* counter,
                                                const int32_t* __restrict__ banned, int seq_arg) {
    __shared__ float sv[4];
    __shared__ int si[4];
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = seq_arg >= 0 ? seq_arg : step->seq;
    const float* logits = logits_base + (size_t)seq * V;
    const int nb = gridDim.x;
    const int per = (V + nb - 1) / nb;
    const int i0 = blockIdx.x * per, i1 = min(V, i0 + per);
    float bv = -INFINITY; int bi = 0x7fffffff;
    const int32_t* ban = banned + (size_t)seq * (1 + BAN_MAX);
    const int nban = ban[0];
    for (int i = i0 + tid; i < i1; i += 256) {
        bool allowed = true;
        for (int k = 0; k < nban; ++k) allowed = allowed && i != ban[1 + k];
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
        st[seq].next_token = bi;
        *counter = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

static int g_gemv_grid = 256;       // workgroups per matrix-vector kernel; decode_init sets it to the number of compute units
static size_t g_gemv_lds_limit = 48 * 1024;   // dynamic LDS a matrix-vector kernel may ask for (raised by decode_init)

template <typename WT, int EPI, int NB>
static hipError_t launch_gemv_n(const GemvArgs& a, size_t lds, const Geom& g, hipStream_t s) {
    hipLaunchKernelGGL((k_gemv<WT, EPI, NB>), dim3(g_gemv_grid), dim3(256), lds, s, a, g);
    return hipGetLastError();
}

// Early request of the vector when it is a plain one that fits one batch: 4 or 8 x 16 bytes per thread (with as
// many of the gain) in the normalising products, 4 or 16 in the residual ones.
template <int EPI> struct EarlyNB { static constexpr int SMALL = 4, LARGE = EPI == EPI_RESID ? 16 : 8, HUGE = 32; };

template <typename WT, int EPI>
static hipError_t launch_gemv_t(const GemvArgs& a0, const Geom& g, hipStream_t s) {
    GemvArgs a = a0;
    const int grid = g_gemv_grid;
    a.done_cap = (a.units + grid * 4 - 1) / (grid * 4) + 1;
    const int kg = a.K / Elem<WT>::EPL, kt = (kg + 255) / 256;
    const size_t lds = (size_t)(kt * 256 + 64) * Elem<WT>::EPL * sizeof(float) + (size_t)4 * a.done_cap * sizeof(float4);
    if (lds > g_gemv_lds_limit) return hipErrorInvalidValue;
    if (EPI != EPI_RESID && !(a.x && a.gain)) return hipErrorInvalidValue;   // the normalising products take a vector and a gain
    if (EPI == EPI_RESID && a.gain) return hipErrorInvalidValue;
    if (a.x && a.K <= 1024 * EarlyNB<EPI>::SMALL) return launch_gemv_n<WT, EPI, EarlyNB<EPI>::SMALL>(a, lds, g, s);
    if (a.x && a.K <= 1024 * EarlyNB<EPI>::LARGE) return launch_gemv_n<WT, EPI, EarlyNB<EPI>::LARGE>(a, lds, g, s);
    if (EPI == EPI_RESID && a.x && a.K <= 1024 * EarlyNB<EPI>::HUGE) return launch_gemv_n<WT, EPI_RESID, EarlyNB<EPI_RESID>::HUGE>(a, lds, g, s);
    return launch_gemv_n<WT, EPI, 0>(a, lds, g, s);
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

template <typename WT, int EPI>
static hipError_t set_lds_t(int bytes) {
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, 0>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, EarlyNB<EPI>::SMALL>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if ((e = hipFuncSetAttribute((const void*)(k_gemv<WT, EPI, EarlyNB<EPI>::LARGE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))) return e;
    if (EPI != EPI_RESID) return hipSuccess;
    return hipFuncSetAttribute((const void*)(k_gemv<WT, EPI_RESID, EarlyNB<EPI_RESID>::HUGE>), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
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
    if (bytes <= 48 * 1024) return hipSuccess;
    g_gemv_lds_limit = (size_t)bytes;
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
    return hipSuccess;
}

static hipError_t launch_gemv(int dtype, int epi, const GemvArgs& a, const Geom& g, hipStream_t s) {
    return dtype == 0 ? launch_gemv_w<float>(epi, a, g, s) : launch_gemv_w<bf16_t>(epi, a, g, s);
}

hipError_t launch_begin_step(const DecodeBuffers& b, int seq, int forced, int32_t* token_early, hipStream_t s) {
    hipLaunchKernelGGL(k_begin_step, dim3(1), dim3(64), 0, s, b.step, b.seq_state, seq, forced, b.token_log, token_early);
    return hipGetLastError();
}

hipError_t launch_embed(int dtype, const void* E, const DecodeBuffers& b, const Geom& g, hipStream_t s) {
    const int grid = (g.d + 255) / 256;
    if (dtype == 0) hipLaunchKernelGGL(k_embed<float>, dim3(grid), dim3(256), 0, s, (const float*)E, b.step, b.x, g.d);
    else hipLaunchKernelGGL(k_embed<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)E, b.step, b.x, g.d);
    return hipGetLastError();
}

hipError_t launch_qkv(int dtype, const void* wqkv, const float* gain, void* kv_layer, const DecodeBuffers& b,
                      const Geom& g, hipStream_t s) {
    GemvArgs a{};
    a.W = wqkv; a.rows = (g.Hq + 2 * g.Hkv) * g.dh; a.K = g.d; a.units = a.rows / 2;
    a.x = b.x; a.gain = gain; a.q_out = b.q; a.kv_layer = kv_layer;
    a.rope_cos = b.rope_cos; a.rope_sin = b.rope_sin; a.step = b.step;
    return launch_gemv(dtype, EPI_QKV, a, g, s);
}

hipError_t launch_oproj(int dtype, const void* wo, int merge_nsplit, const DecodeBuffers& b, const Geom& g, hipStream_t s) {
    GemvArgs a{};
    a.W = wo; a.rows = g.d; a.K = g.Hq * g.dh; a.units = (a.rows + 1) / 2;
    a.x = b.o; a.gain = nullptr; a.y = b.x; a.res = b.x; a.step = b.step;
    if (merge_nsplit > 0) {
        if (merge_nsplit > MERGE_MAX_SPLIT) return hipErrorInvalidValue;
        a.x = nullptr; a.part_acc = b.part_acc; a.part_ml = b.part_ml;
        a.merge_nsplit = merge_nsplit; a.merge_dh = g.dh; a.merge_hq = g.Hq;
    }
    return launch_gemv(dtype, EPI_RESID, a, g, s);
}

hipError_t launch_gateup(int dtype, const void* wgu, const float* gain, const DecodeBuffers& b, const Geom& g, hipStream_t s) {
    GemvArgs a{};
    a.W = wgu; a.rows = 2 * g.F; a.K = g.d; a.units = g.F;
    a.x = b.x; a.gain = gain; a.y = b.a; a.step = b.step;
    return launch_gemv(dtype, EPI_SWIGLU, a, g, s);
}

hipError_t launch_down(int dtype, const void* wd, const DecodeBuffers& b, const Geom& g, hipStream_t s) {
    GemvArgs a{};
    a.W = wd; a.rows = g.d; a.K = g.F; a.units = (a.rows + 1) / 2;
    a.x = b.a; a.gain = nullptr; a.y = b.x; a.res = b.x; a.step = b.step;
    return launch_gemv(dtype, EPI_RESID, a, g, s);
}

hipError_t launch_lmhead(int dtype, const void* wout, const float* gain, float* logits, const DecodeBuffers& b,
                         const Geom& g, hipStream_t s) {
    GemvArgs a{};
    a.W = wout; a.rows = g.V; a.K = g.d; a.units = (a.rows + 1) / 2;
    a.x = b.x; a.gain = gain; a.y = logits; a.step = b.step;
    return launch_gemv(dtype, EPI_STORE, a, g, s);
}

template <typename KVT, int DH, bool PAIR>
static hipError_t launch_attn_t(const AttnArgs& a, const Geom& g, hipStream_t s) {
    const dim3 grid(g.Hkv, a.nsplit), block(256);
#define ATTN_CASE(GG)                                                                                                   \
    case GG: {                                                                                                          \
        const size_t lds = sizeof(float) * attn_lds_floats<KVT, DH, GG>();                                              \
        if (lds > 48 * 1024) {                                                                                          \
            hipError_t e = hipFuncSetAttribute((const void*)(k_attn_decode<KVT, DH, GG, PAIR>),                         \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                   \
            if (e) return e;                                                                                            \
        }                                                                                                               \
        hipLaunchKernelGGL((k_attn_decode<KVT, DH, GG, PAIR>), grid, block, lds, s, a, g);                              \
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
                              const Geom& g, hipStream_t s) {
    AttnArgs a{};
    a.defer_merge = merge_in_oproj ? 1 : 0;
    a.q = b.q; a.kv_layer = kv_layer; a.step = b.step; a.o = b.o;
    a.part_acc = b.part_acc; a.part_ml = b.part_ml; a.counters = b.attn_counters; a.nsplit = nsplit;
    if (dtype == 0) return g.dh == 64 ? launch_attn_t<float, 64, false>(a, g, s) : launch_attn_t<float, 128, false>(a, g, s);
    if (g.kv_lo_offset) return g.dh == 64 ? launch_attn_t<bf16_t, 64, true>(a, g, s) : launch_attn_t<bf16_t, 128, true>(a, g, s);
    return g.dh == 64 ? launch_attn_t<bf16_t, 64, false>(a, g, s) : launch_attn_t<bf16_t, 128, false>(a, g, s);
}

hipError_t launch_argmax(const float* logits_base, const DecodeBuffers& b, const Geom& g, hipStream_t s, int seq) {
    int nb = (g.V + 2047) / 2048;
    if (nb > ARGMAX_MAX_BLOCKS) nb = ARGMAX_MAX_BLOCKS;
    hipLaunchKernelGGL(k_argmax, dim3(nb), dim3(256), 0, s, logits_base, g.V, b.step, b.seq_state, b.amax_v, b.amax_i, b.amax_counter, b.banned, seq);
    return hipGetLastError();
}

}  // namespace asynclm
