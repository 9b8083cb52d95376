// One decoding step as ONE persistent kernel (gfx950): every workgroup owns a fixed share of the rows
// of every matrix, phases are separated by grid-wide barriers, and the first weight tiles of the next
// phase are requested before each barrier, so that HBM keeps streaming while the workgroups wait.
//
// Launch: cooperative, one workgroup of 256 threads (4 waves) per compute unit.
// Phases per layer:  QKV (+norm, rotary, K/V write) | attention partials | merge of the splits |
//                    O (+residual) | gate/up (+norm, SwiGLU) | down (+residual);
// then final norm + output head with a running argmax, and the argmax merge by workgroup 0.
//
// A wave walks its rows pair by pair ("units", see decode_device.h) in tiles of 2 rows x 4 k-steps
// (8 loads of 16 bytes per lane = 8 KiB per wave) through a ring of four register tiles: while one
// tile is multiplied, the next three are in flight.  The loop body has no conditional code around the
// loads or their use (tiles past the end re-read the last tile and are multiplied by zeros), because
// the compiler otherwise sinks the loads next to their users and the pipeline collapses.
#include "common.h"
#include "launch.h"
#include "decode_device.h"

#include <algorithm>

namespace asynclm {

constexpr unsigned BARRIER_SPIN_LIMIT = 1u << 22;   // polls before a workgroup gives up (about a second)

struct FusedLayer {
    const float* attn_norm; const void* wqkv; const void* wo;
    const float* ffn_norm; const void* wgate_up; const void* wdown;
    void* kv_layer;
};

struct FusedArgs {
    const FusedLayer* layers;
    int32_t n_layers;
    const void* embed; const float* final_norm; const void* lm_head;
    Geom g;
    SeqState* seq_state;
    int32_t seq, forced, with_head;
    int32_t* token_log;
    float *x, *q, *o, *a, *part_acc, *part_ml, *logits;
    const float *rope_cos, *rope_sin;
    float* amax_v; int32_t* amax_i;
    unsigned* bar;          // grid barrier state (see grid_arrive)
    int32_t nsplit;         // attention splits per kv head (<= gridDim.x / Hkv)
    int32_t merge_in_stage; // 1: the O projection merges the splits while staging (nsplit <= MERGE_MAX_SPLIT), no merge phase
    int32_t xs_groups;      // LDS capacity of the staged vector, in groups of EPL elements
    int32_t done_cap;       // units one wave can park in LDS before its epilogues run
    unsigned long long* trace;   // optional [stamp][workgroup]: the 100 MHz wall clock at every phase boundary
};

// ---------------------------------------------------------------------------------------------
// grid barrier
// ---------------------------------------------------------------------------------------------

// One flag per workgroup instead of one shared counter: arrivals are plain stores to different
// addresses (an atomic counter would serialise the 256 arrivals at the memory side), and a waiting
// workgroup reads all flags with one load per lane.  bar[0] = epoch of the last barrier of the previous
// launch, bar[1] = error flag, bar[BAR_FLAGS + w] = last epoch workgroup w has reached.
constexpr int BAR_FLAGS = 8;

// Arrive at barrier `epoch`.  All global stores of the workgroup made before the call are visible to
// every workgroup that later passes grid_wait(epoch).
__device__ __forceinline__ void grid_arrive(unsigned* bar, unsigned epoch) {
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_store(&bar[BAR_FLAGS + blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Wait until every workgroup has arrived at `epoch`.  Returns false (for the whole workgroup) when the
// spin limit is hit or another workgroup has already given up; the caller then leaves the kernel.
__device__ __forceinline__ bool grid_wait(unsigned* bar, unsigned epoch, int* s_flag, int32_t* token_log) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x, nwg = gridDim.x;
        unsigned spins = 0;
        int ok = 1;
        for (;;) {
            bool mine = true;
            for (int w = lane; w < nwg; w += 64)
                mine = mine && (int)(__hip_atomic_load(&bar[BAR_FLAGS + w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) >= 0;
            if (__all(mine)) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > BARRIER_SPIN_LIMIT || __hip_atomic_load(&bar[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                ok = 0;
                break;
            }
        }
        if (lane == 0) {
            if (!ok) { atomicExch(&bar[1], 1u); token_log[1] = 1; }    // token_log[1]: read back by the host with the token
            *s_flag = ok;
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return *s_flag != 0;
}

// ---------------------------------------------------------------------------------------------
// matrix-vector phase
// ---------------------------------------------------------------------------------------------

// ---------------------------------------------------------------------------------------------
// the step
// ---------------------------------------------------------------------------------------------

#define FUSED_TRACE() do { if (a.trace && threadIdx.x == 0) a.trace[(size_t)(ntrace++) * gridDim.x + blockIdx.x] = wall_clock64(); } while (0)

template <typename WT, int DH, int G, bool PAIR>
__global__ __launch_bounds__(256) void k_decode_fused(FusedArgs a) {
    int ntrace = 0;
    constexpr int EPL = Elem<WT>::EPL;
    extern __shared__ float4 lds4[];
    __shared__ float red[4];
    __shared__ int s_flag;
    __shared__ float s_bv[4];
    __shared__ int s_bi[4];

    const Geom& g = a.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwg = gridDim.x;
    const int plane_stride = a.xs_groups;
    float4* xs = lds4;
    float* attn_lds = reinterpret_cast<float*>(lds4);    // the attention reuses the staged-vector area
    float* mf = reinterpret_cast<float*>(lds4);          // merge phase scratch
    float4* done = lds4 + (size_t)plane_stride * (EPL / 4) + (size_t)wave * a.done_cap;   // finished units of this wave

    unsigned target = __hip_atomic_load(&a.bar[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // epoch counter
    const SeqState st = a.seq_state[a.seq];
    const int pos = st.len;
    const int token = a.forced >= 0 ? a.forced : st.next_token;

    // residual stream of the new row: x = E[token]
    {
        const WT* erow = (const WT*)a.embed + (size_t)token * g.d;
        for (int i = blockIdx.x * 256 + tid; i < g.d; i += nwg * 256) a.x[i] = Elem<WT>::load1(erow + i);
    }

    const int n_qkv = (g.Hq + 2 * g.Hkv) * g.dh, qd = g.Hq * g.dh;
    Slot ring[RING];
    Cursor lc;
    float best_v = -INFINITY; int best_i = 0x7fffffff;
    EpiOut eo;
    eo.rope_cos = a.rope_cos; eo.rope_sin = a.rope_sin; eo.pos = pos; eo.seq = a.seq; eo.q_out = a.q;

    Phase<WT> ph = make_phase<WT, EPI_QKV>(a.layers[0].wqkv, n_qkv, g.d, n_qkv / 2);
    grid_arrive(a.bar, target + 1);
    phase_prefetch<WT, EPI_QKV>(ring, ph, lc, lane, g, eo);
    target += 1;
    if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();

    for (int l = 0; l < a.n_layers; ++l) {
        const FusedLayer L = a.layers[l];
        // ---- QKV: x -> q, K/V cache row `pos`
        {
            const float ss = stage_vector<WT>(xs, plane_stride, VecSource{a.x, L.attn_norm}, g.d, ph.Kg, ph.KT, true, red);
            eo.kv_layer = L.kv_layer; eo.rows = n_qkv;
            phase_run<WT, EPI_QKV>(ring, ph, lc, xs, plane_stride, rsqrtf(ss / (float)g.d + g.eps), eo, g, lane, done, best_v, best_i);
        }
        ph = make_phase<WT, EPI_RESID>(L.wo, g.d, qd, (g.d + 1) / 2);
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        // O-projection tiles: held in registers across the attention.  Their residual operands are x, which
        // no phase writes before the O projection itself.
        eo.y = a.x; eo.res = a.x; eo.rows = g.d;
        phase_prefetch<WT, EPI_RESID>(ring, ph, lc, lane, g, eo);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();

        // ---- attention partials: workgroup = (kv head, split)
        {
            const int kvh = blockIdx.x % g.Hkv, split = blockIdx.x / g.Hkv, nsplit = a.nsplit;
            if (split < nsplit) {
                constexpr int PPW = 64 / (DH / EPL);
                const int len = pos + 1, quantum = 4 * PPW;
                int per = (len + nsplit - 1) / nsplit;
                per = (per + quantum - 1) / quantum * quantum;
                const int s0 = min(split * per, len), s1 = min(s0 + per, len);
                const WT* Kp = (const WT*)L.kv_layer + (size_t)a.seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
                float mh[G], lh[G];
                attn_split<WT, DH, G, PAIR>(a.q, Kp, Kp + g.kv_v_offset, g.kv_lo_offset, kvh, s0, s1, g.scale, attn_lds, mh, lh);
                for (int t = tid; t < G * DH; t += 256) {
                    const int h = t / DH, dim = t - h * DH, hq = kvh * G + h;
                    const float A = attn_gather<WT, DH, G>(attn_lds, h, dim);
                    float M = mh[0], Ls = lh[0];
#pragma unroll
                    for (int hh = 1; hh < G; ++hh) if (hh == h) { M = mh[hh]; Ls = lh[hh]; }
                    a.part_acc[((size_t)hq * nsplit + split) * DH + dim] = A;
                    if (dim == 0) { a.part_ml[((size_t)hq * nsplit + split) * 2] = M; a.part_ml[((size_t)hq * nsplit + split) * 2 + 1] = Ls; }
                }
            }
            __syncthreads();            // LDS is reused by the next phase
        }
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();

        // ---- merge of the splits: thread = (query head, 4 channels, one eighth of the splits)
        if (!a.merge_in_stage) {
            constexpr int TPH = DH * 2;                     // threads per head
            constexpr int HPW = 256 / TPH;                  // heads per workgroup
            const int nsplit = a.nsplit;
            const int hl = tid / TPH, within = tid - hl * TPH, d4 = within >> 3, grp = within & 7;
            const int hq = blockIdx.x * HPW + hl;
            const bool active = blockIdx.x * HPW < g.Hq;    // uniform per workgroup
            if (active) {
                for (int t = tid; t < HPW * nsplit; t += 256) {
                    const int h2 = t / nsplit, sp = t - h2 * nsplit, hh = blockIdx.x * HPW + h2;
                    if (hh < g.Hq) {
                        mf[h2 * 2 * ATTN_MAX_SPLIT + sp] = a.part_ml[((size_t)hh * nsplit + sp) * 2];
                        mf[h2 * 2 * ATTN_MAX_SPLIT + ATTN_MAX_SPLIT + sp] = a.part_ml[((size_t)hh * nsplit + sp) * 2 + 1];
                    }
                }
                __syncthreads();
                if (tid < HPW && blockIdx.x * HPW + tid < g.Hq) {
                    float* fm = mf + tid * 2 * ATTN_MAX_SPLIT;
                    float M = -INFINITY, Ls = 0.f;
                    for (int sp = 0; sp < nsplit; ++sp) M = fmaxf(M, fm[sp]);
                    for (int sp = 0; sp < nsplit; ++sp) {
                        const float f = fm[sp] > -INFINITY ? expf(fm[sp] - M) : 0.f;
                        Ls += fm[ATTN_MAX_SPLIT + sp] * f;
                        fm[sp] = f;
                    }
                    const float inv = 1.f / Ls;
                    for (int sp = 0; sp < nsplit; ++sp) fm[sp] *= inv;
                }
                __syncthreads();
                float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
                if (hq < g.Hq) {
                    const float4* src = (const float4*)(a.part_acc + (size_t)hq * nsplit * DH) + d4;
                    const float* fm = mf + hl * 2 * ATTN_MAX_SPLIT;
#pragma unroll 4
                    for (int sp = grp; sp < nsplit; sp += 8) {
                        const float4 v = src[(size_t)sp * (DH / 4)];
                        const float f = fm[sp];
                        r.x = fmaf(v.x, f, r.x); r.y = fmaf(v.y, f, r.y); r.z = fmaf(v.z, f, r.z); r.w = fmaf(v.w, f, r.w);
                    }
                }
#pragma unroll
                for (int o = 1; o < 8; o <<= 1) {
                    r.x += __shfl_xor(r.x, o, 64); r.y += __shfl_xor(r.y, o, 64);
                    r.z += __shfl_xor(r.z, o, 64); r.w += __shfl_xor(r.w, o, 64);
                }
                if (hq < g.Hq && grp == 0) ((float4*)(a.o + (size_t)hq * DH))[d4] = r;
            }
        }
        FUSED_TRACE();
        if (!a.merge_in_stage) {
            grid_arrive(a.bar, target + 1);
            target += 1;
            if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
        }
        FUSED_TRACE();

        // ---- O projection + residual (tiles were requested before the attention)
        {
            VecSource vs{a.o, nullptr};
            if (a.merge_in_stage) { vs.x = nullptr; vs.part_acc = a.part_acc; vs.part_ml = a.part_ml; vs.nsplit = a.nsplit; vs.DH = DH; vs.Hq = g.Hq; }
            stage_vector<WT>(xs, plane_stride, vs, qd, ph.Kg, ph.KT, true, red);
            eo.y = a.x; eo.res = a.x; eo.rows = g.d;
            phase_run<WT, EPI_RESID>(ring, ph, lc, xs, plane_stride, 1.f, eo, g, lane, done, best_v, best_i);
        }
        ph = make_phase<WT, EPI_SWIGLU>(L.wgate_up, 2 * g.F, g.d, g.F);
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        phase_prefetch<WT, EPI_SWIGLU>(ring, ph, lc, lane, g, eo);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();

        // ---- gate/up + SwiGLU
        {
            const float ss = stage_vector<WT>(xs, plane_stride, VecSource{a.x, L.ffn_norm}, g.d, ph.Kg, ph.KT, true, red);
            eo.y = a.a; eo.rows = 2 * g.F;
            phase_run<WT, EPI_SWIGLU>(ring, ph, lc, xs, plane_stride, rsqrtf(ss / (float)g.d + g.eps), eo, g, lane, done, best_v, best_i);
        }
        ph = make_phase<WT, EPI_RESID>(L.wdown, g.d, g.F, (g.d + 1) / 2);
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        eo.y = a.x; eo.res = a.x; eo.rows = g.d;
        phase_prefetch<WT, EPI_RESID>(ring, ph, lc, lane, g, eo);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();

        // ---- down projection + residual
        {
            stage_vector<WT>(xs, plane_stride, VecSource{a.a, nullptr}, g.F, ph.Kg, ph.KT, true, red);
            eo.y = a.x; eo.res = a.x; eo.rows = g.d;
            phase_run<WT, EPI_RESID>(ring, ph, lc, xs, plane_stride, 1.f, eo, g, lane, done, best_v, best_i);
        }
        const bool more = l + 1 < a.n_layers;
        if (more) ph = make_phase<WT, EPI_QKV>(a.layers[l + 1].wqkv, n_qkv, g.d, n_qkv / 2);
        else ph = make_phase<WT, EPI_STORE>(a.lm_head, g.V, g.d, (g.V + 1) / 2);
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        if (more) phase_prefetch<WT, EPI_QKV>(ring, ph, lc, lane, g, eo);
        else if (a.with_head) phase_prefetch<WT, EPI_STORE>(ring, ph, lc, lane, g, eo);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();
    }

    if (a.with_head) {
        const float ss = stage_vector<WT>(xs, plane_stride, VecSource{a.x, a.final_norm}, g.d, ph.Kg, ph.KT, true, red);
        eo.y = a.logits; eo.rows = g.V;
        best_v = -INFINITY; best_i = 0x7fffffff;
        phase_run<WT, EPI_STORE>(ring, ph, lc, xs, plane_stride, rsqrtf(ss / (float)g.d + g.eps), eo, g, lane, done, best_v, best_i);
        if (lane == 0) { s_bv[wave] = best_v; s_bi[wave] = best_i; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w) amax_merge(best_v, best_i, s_bv[w], s_bi[w]);
            a.amax_v[blockIdx.x] = best_v; a.amax_i[blockIdx.x] = best_i;
        }
        FUSED_TRACE();
        grid_arrive(a.bar, target + 1);
        target += 1;
        if (!grid_wait(a.bar, target, &s_flag, a.token_log)) return;
    FUSED_TRACE();
    }

    if (blockIdx.x != 0) return;
    int next = st.next_token;
    if (a.with_head) {
        float bv = -INFINITY; int bi = 0x7fffffff;
        for (int b = tid; b < nwg; b += 256) amax_merge(bv, bi, a.amax_v[b], a.amax_i[b]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
            amax_merge(bv, bi, ov, oi);
        }
        __syncthreads();
        if (lane == 0) { s_bv[wave] = bv; s_bi[wave] = bi; }
        __syncthreads();
        if (tid == 0) for (int w = 1; w < 4; ++w) amax_merge(bv, bi, s_bv[w], s_bi[w]);
        next = bi;
    }
    if (tid == 0) {
        a.seq_state[a.seq].len = pos + 1;
        a.seq_state[a.seq].next_token = next;
        *a.token_log = token;
        __hip_atomic_store(&a.bar[0], target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

typedef void (*fused_kernel_t)(FusedArgs);

static fused_kernel_t pick_kernel(int dtype, const Geom& g) {
    const int G = g.Hq / g.Hkv;
    const bool pair = g.kv_lo_offset != 0;
    if (dtype == 0) {
        if (g.dh == 64 && G == 1) return k_decode_fused<float, 64, 1, false>;
        return nullptr;
    }
    if (g.dh != 128) return nullptr;
    if (G == 4) return pair ? k_decode_fused<bf16_t, 128, 4, true> : k_decode_fused<bf16_t, 128, 4, false>;
    if (G == 8) return pair ? k_decode_fused<bf16_t, 128, 8, true> : k_decode_fused<bf16_t, 128, 8, false>;
    return nullptr;
}

// LDS bytes: the staged vector (largest K of any phase, padded to whole tiles plus a block of zeros),
// which the attention phases reuse, then per wave one float4 per unit of its largest phase.
static size_t fused_lds_bytes(int dtype, const Geom& g, int grid, int* xs_groups, int* done_cap) {
    const int epl = dtype == 0 ? 4 : 8;
    const int kmax = std::max(std::max(g.d, g.F), g.Hq * g.dh);
    const int kg = kmax / epl, kt = (kg + 255) / 256;
    *xs_groups = kt * 256 + 64;
    size_t bytes = (size_t)(*xs_groups) * epl * sizeof(float);
    const int G = g.Hq / g.Hkv, ppw = 64 / (g.dh / epl);
    const size_t attn = sizeof(float) * (size_t)(ATTN_CHUNK * G + 4 * G + 4 * ppw * G * g.dh);
    bytes = std::max(bytes, attn);
    const int units_max = std::max(std::max((g.Hq + 2 * g.Hkv) * g.dh / 2, g.F), (g.V + 1) / 2);
    *done_cap = (units_max + grid * 4 - 1) / (grid * 4) + 1;
    return bytes + (size_t)4 * (*done_cap) * sizeof(float4);
}

hipError_t fused_init(int dtype, const Geom& g, FusedPlan* plan) {
    plan->supported = false;
    fused_kernel_t k = pick_kernel(dtype, g);
    if (!k) return hipSuccess;
    int dev = 0, cus = 0, coop = 0;
    hipError_t e;
    if ((e = hipGetDevice(&dev))) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) return e;
    if ((e = hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev))) return e;
    if (!coop || cus < g.Hkv || cus > ARGMAX_MAX_BLOCKS) return hipSuccess;
    plan->lds_bytes = fused_lds_bytes(dtype, g, cus, &plan->xs_groups, &plan->done_cap);
    if (plan->lds_bytes > 160 * 1024) return hipSuccess;
    if ((e = hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)plan->lds_bytes))) return e;
    int per_cu = 0;
    if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)k, 256, plan->lds_bytes))) return e;
    if (per_cu < 1) return hipSuccess;
    plan->grid = cus;
    plan->nsplit = std::min(cus / g.Hkv, (int)ATTN_MAX_SPLIT);
    // the merge phase needs one workgroup per query head (two heads per workgroup at head_dim 64)
    if (cus * (256 / (g.dh * 2)) < g.Hq) return hipSuccess;
    plan->supported = true;
    return hipSuccess;
}

hipError_t launch_decode_fused(int dtype, const FusedPlan& plan, const FusedLaunch& L, const DecodeBuffers& b, const Geom& g,
                               hipStream_t s) {
    fused_kernel_t k = pick_kernel(dtype, g);
    if (!k || !plan.supported) return hipErrorInvalidValue;
    FusedArgs a{};
    a.layers = (const FusedLayer*)L.layers_dev; a.n_layers = L.n_layers;
    a.embed = L.embed; a.final_norm = L.final_norm; a.lm_head = L.lm_head;
    a.g = g; a.seq_state = b.seq_state; a.seq = L.seq; a.forced = L.forced; a.with_head = L.with_head ? 1 : 0;
    a.token_log = b.token_log;
    a.x = b.x; a.q = b.q; a.o = b.o; a.a = b.a; a.part_acc = b.part_acc; a.part_ml = b.part_ml; a.logits = L.logits;
    a.rope_cos = b.rope_cos; a.rope_sin = b.rope_sin; a.amax_v = b.amax_v; a.amax_i = b.amax_i;
    a.bar = L.bar; a.nsplit = L.nsplit; a.merge_in_stage = L.merge_in_stage ? 1 : 0;
    if (L.nsplit < 1 || L.nsplit > plan.nsplit || (L.merge_in_stage && L.nsplit > MERGE_MAX_SPLIT)) return hipErrorInvalidValue;
    a.xs_groups = plan.xs_groups; a.done_cap = plan.done_cap; a.trace = (unsigned long long*)L.trace;
    void* params[] = {&a};
    return hipLaunchCooperativeKernel((const void*)k, dim3(plan.grid), dim3(256), params, (unsigned)plan.lds_bytes, s);
}

static_assert(sizeof(FusedLayer) == 7 * sizeof(void*), "FusedLayer is uploaded as 7 pointers per layer");

}  // namespace asynclm
