// Device code shared by the per-kernel decode path and the fused (persistent) decode step:
// row-pair mapping and epilogues of the matrix-vector products, the split-sequence attention
// of one workgroup, argmax merging.
#pragma once

#include "common.h"
#include "launch.h"

namespace asynclm {

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };

// Cache write: fp32 as is; bf16 as the rounded value, plus the rounded remainder in the lo plane
// when the cache has one.
// Written through (device-coherent stores): the attention of the same step may already be running on
// another stream when the row is written.
__device__ __forceinline__ void kv_store(float* p, float v, size_t) { store_coherent(p, v); }
__device__ __forceinline__ void kv_store(bf16_t* p, float v, size_t lo_offset) {
    const bf16_t hi = f32_to_bf16(v);
    store_coherent(p, hi);
    if (lo_offset) store_coherent(p + lo_offset, f32_to_bf16(v - __uint_as_float((uint32_t)hi << 16)));
}

// A "unit" is the pair of matrix rows one wave reduces together:
//   STORE / RESID: rows 2u, 2u+1;  SWIGLU: gate row u and up row F+u;  QKV: the two halves
//   (i, i+dh/2) of a rotary pair of one head.
template <int EPI>
__device__ __forceinline__ void unit_rows(int u, int rows, const Geom& g, int& rA, int& rB) {
    if (EPI == EPI_SWIGLU) { rA = u; rB = g.F + u; }
    else if (EPI == EPI_QKV) {
        const int hs = g.dh == 128 ? 6 : 5, half = 1 << hs;      // head_dim is 64 or 128
        const int h = u >> hs, i = u & (half - 1);
        rA = h * g.dh + i; rB = rA + half;
    } else { rA = 2 * u; rB = min(2 * u + 1, rows - 1); }
}

// Where the results of a product go.
struct EpiOut {
    float* y;               // STORE: y[rows]; RESID: y[r] = res[r] + acc; SWIGLU: y[F]
    const float* res;
    float* q_out;           // QKV: rotated queries [Hq*dh]
    void* kv_layer;         // QKV: this layer's K plane of sequence 0
    const float* rope_cos;  // [max_pos][dh/2]
    const float* rope_sin;
    int32_t rows;
    int32_t pos, seq;       // QKV: position and sequence of the row being processed
};

__device__ __forceinline__ void amax_merge(float& bv, int& bi, float v, int i) {
    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

// ---------------------------------------------------------------------------------------------
// split-sequence decode attention of one workgroup (256 threads)
// ---------------------------------------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over groups of N consecutive lanes (N = 8, 16 or 32); every lane of a group gets the total.
// Lane exchanges inside a row of 16 are DPP modifiers of the add (no LDS traffic).
template <int N>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_move<0xB1>(v);                 // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);                 // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);                // row_half_mirror: the other quad of each 8 lanes
    if (N >= 16) v += dpp_move<0x140>(v);   // row_mirror: the other half of the row
    if (N >= 32) v += __shfl_xor(v, 16, 64);
    return v;
}

__device__ __forceinline__ float wave_max_all(float v) {
    v = fmaxf(v, dpp_move<0xB1>(v)); v = fmaxf(v, dpp_move<0x4E>(v));
    v = fmaxf(v, dpp_move<0x141>(v)); v = fmaxf(v, dpp_move<0x140>(v));
    float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

__device__ __forceinline__ float wave_sum_all(float v) {
    v += dpp_move<0xB1>(v); v += dpp_move<0x4E>(v); v += dpp_move<0x141>(v); v += dpp_move<0x140>(v);
    float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

constexpr int ATTN_CHUNK = 256;     // positions whose scores are held in LDS at a time (one per thread)

// LDS floats the attention of one workgroup needs
template <typename KVT, int DH, int G>
__host__ __device__ constexpr int attn_lds_floats() {
    return ATTN_CHUNK * G + 4 * G + 4 * (64 / (DH / Elem<KVT>::EPL)) * G * DH;
}

// Positions [s0, s1) of one kv head for its G query heads.
// q: [Hq*DH] rotated, unscaled.  Kp / Vp: row-major planes of this kv head (row = position); lo_offset: distance
// to the lo planes (PAIR).  Three passes per chunk of up to ATTN_CHUNK positions:
//   1. scores: a group of LPR lanes covers one cached key (16 bytes per lane), the G heads reuse the load,
//      dot products are reduced inside the group with DPP adds, and land in LDS;
//   2. softmax statistics of the chunk, one position per thread (running max m and sum l are replicated);
//   3. P V: the same lane groups walk the values, the probabilities come from LDS.
// On return (after a __syncthreads) lds holds NPART = 4 * PPW partial accumulators [part][G][DH] starting at
// attn_part_offset, all relative to the same maximum; m_out[h], l_out[h] are valid in every thread.
template <typename KVT, int DH, int G, bool PAIR>
__device__ __forceinline__ void attn_split(const float* __restrict__ q, const KVT* __restrict__ Kp,
                                           const KVT* __restrict__ Vp, size_t lo_offset, int kvh, int s0, int s1,
                                           float scale, float* lds, float (&m_out)[G], float (&l_out)[G]) {
    constexpr int EPL = Elem<KVT>::EPL;
    constexpr int LPR = DH / EPL;       // lanes that cover one cached row
    constexpr int PPW = 64 / LPR;       // positions per wave-wide load
    constexpr int PPR = 4 * PPW;        // positions per workgroup-wide round
    constexpr int UN = 4;               // rounds whose loads are issued together
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, c = lane % LPR;
    float* sc = lds;                            // [ATTN_CHUNK][G] scores, then probabilities
    float* wred = lds + ATTN_CHUNK * G;         // [4][G] per-wave partial max / sum
    float* part = wred + 4 * G;                 // [4 * PPW][G][DH]

    float qr[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float* qp = q + (kvh * G + h) * DH + c * EPL;
#pragma unroll
        for (int e4 = 0; e4 < EPL; e4 += 4) {
            const uint4 t = load16(qp + e4);
            qr[h][e4] = __uint_as_float(t.x) * scale; qr[h][e4 + 1] = __uint_as_float(t.y) * scale;
            qr[h][e4 + 2] = __uint_as_float(t.z) * scale; qr[h][e4 + 3] = __uint_as_float(t.w) * scale;
        }
    }
    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    for (int c0 = s0; c0 < s1; c0 += ATTN_CHUNK) {
        const int c1 = min(c0 + ATTN_CHUNK, s1), nc = c1 - c0;
        // ---- 1. scores
        for (int r0 = 0; r0 < nc; r0 += PPR * UN) {
            uint4 kr[UN], krl[PAIR ? UN : 1];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int p = min(c0 + r0 + u * PPR + wave * PPW + sub, s1 - 1);
                kr[u] = load16(Kp + (size_t)p * DH + c * EPL);
                if (PAIR) krl[u] = load16(Kp + lo_offset + (size_t)p * DH + c * EPL);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int pl = r0 + u * PPR + wave * PPW + sub;      // position within the chunk
                float kf[EPL];
                Elem<KVT>::expand(kr[u], kf);
                if (PAIR) {
                    float kl[EPL];
                    Elem<KVT>::expand(krl[u], kl);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) kf[e] += kl[e];
                }
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float s = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) s = fmaf(qr[h][e], kf[e], s);
                    s = group_sum<LPR>(s);
                    if (c == 0 && pl < ATTN_CHUNK) sc[pl * G + h] = pl < nc ? s : -INFINITY;
                }
            }
        }
        __syncthreads();
        // ---- 2. statistics: thread t owns position c0 + t
        float sv[G], corr[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            sv[h] = tid < nc ? sc[tid * G + h] : -INFINITY;
            const float wm = wave_max_all(sv[h]);
            if (lane == 0) wred[wave * G + h] = wm;
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float cm = fmaxf(fmaxf(wred[h], wred[G + h]), fmaxf(wred[2 * G + h], wred[3 * G + h]));
            const float mn = fmaxf(m[h], cm);            // finite: the chunk is not empty
            corr[h] = expf(m[h] - mn);                   // exp(-inf) = 0 for the first chunk
            m[h] = mn;
            sv[h] = expf(sv[h] - mn);                    // 0 for threads without a position
        }
        __syncthreads();                                  // every thread has read wred
#pragma unroll
        for (int h = 0; h < G; ++h) {
            if (tid < nc) sc[tid * G + h] = sv[h];
            const float ws = wave_sum_all(sv[h]);
            if (lane == 0) wred[wave * G + h] = ws;
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < G; ++h) {
            l[h] = l[h] * corr[h] + ((wred[h] + wred[G + h]) + (wred[2 * G + h] + wred[3 * G + h]));
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] *= corr[h];
        }
        // ---- 3. P V
        for (int r0 = 0; r0 < nc; r0 += PPR * UN) {
            uint4 vr[UN], vrl[PAIR ? UN : 1];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int p = min(c0 + r0 + u * PPR + wave * PPW + sub, s1 - 1);
                vr[u] = load16(Vp + (size_t)p * DH + c * EPL);
                if (PAIR) vrl[u] = load16(Vp + lo_offset + (size_t)p * DH + c * EPL);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int pl = r0 + u * PPR + wave * PPW + sub;
                float vf[EPL];
                Elem<KVT>::expand(vr[u], vf);
                if (PAIR) {
                    float vl[EPL];
                    Elem<KVT>::expand(vrl[u], vl);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) vf[e] += vl[e];
                }
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float pr = pl < nc ? sc[pl * G + h] : 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(pr, vf[e], acc[h][e]);
                }
            }
        }
        __syncthreads();                                  // sc and wred are rewritten by the next chunk
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m_out[h] = m[h]; l_out[h] = l[h];
#pragma unroll
        for (int e = 0; e < EPL; ++e) part[((wave * PPW + sub) * G + h) * DH + c * EPL + e] = acc[h][e];
    }
    __syncthreads();
}

// Sum of the workgroup's partial accumulators for (head h of the group, channel dim).
template <typename KVT, int DH, int G>
__device__ __forceinline__ float attn_gather(const float* lds, int h, int dim) {
    constexpr int NPART = 4 * (64 / (DH / Elem<KVT>::EPL));
    const float* part = lds + ATTN_CHUNK * G + 4 * G;
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < NPART; ++i) a += part[(i * G + h) * DH + dim];
    return a;
}

// ---------------------------------------------------------------------------------------------
// staging of the input vector of a matrix-vector product
// ---------------------------------------------------------------------------------------------

constexpr int MERGE_MAX_SPLIT = 8;      // attention splits that the O projection can merge while staging

// Where the vector comes from: a plain fp32 vector x (times an optional gain), or - when x is null - the
// attention output formed on the fly from the per-split partial accumulators:
//   o[h][dim] = sum_s f[h][s] * part_acc[h][s][dim],   f[h][s] = exp(m[h][s] - M[h]) / L[h].
struct VecSource {
    const float* x;
    const float* gain;
    const float* part_acc;  // [Hq][nsplit][DH]
    const float* part_ml;   // [Hq][nsplit][2]
    int nsplit, DH, Hq;
};

__device__ __forceinline__ float4 as_float4(const uint4& v) {
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}

// Stages K elements into the planar LDS layout (plane p of group grp holds elements 4p..4p+3 of the group of
// EPL elements; planes are plane_stride float4 apart) and returns the sum of squares of the unscaled vector
// (valid after the trailing __syncthreads).  With `pad`, groups [Kg, 256 KT) and the last 64 groups of each
// plane are zero-filled.
// All loads of a batch are issued before the first is used.
template <typename WT, int NB = 4>
__device__ __forceinline__ float stage_vector(float4* xs, int plane_stride, const VecSource& src, int K, int Kg, int KT,
                                              bool pad, float* red) {
    constexpr int NP = Elem<WT>::EPL / 4;
    const int tid = threadIdx.x, n4 = K >> 2;
    float ss = 0.f;
    if (src.x && src.gain) {
        for (int base = 0; base < n4; base += 1024) {
            float4 v[4], gn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k4 = min(base + j * 256 + tid, n4 - 1);
                v[j] = as_float4(load16(src.x + 4 * (size_t)k4));
                gn[j] = as_float4(load16(src.gain + 4 * (size_t)k4));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k4 = base + j * 256 + tid;
                if (k4 < n4) {
                    ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
                    const int grp = k4 / NP, pl = k4 - grp * NP;
                    xs[pl * plane_stride + grp] = make_float4(v[j].x * gn[j].x, v[j].y * gn[j].y, v[j].z * gn[j].z, v[j].w * gn[j].w);
                }
            }
        }
    } else if (src.x) {
        // no gain: NB loads per thread are in flight at once (a long vector costs few memory round trips)
        for (int base = 0; base < n4; base += NB * 256) {
            float4 v[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) v[j] = as_float4(load16(src.x + 4 * (size_t)min(base + j * 256 + tid, n4 - 1)));
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int k4 = base + j * 256 + tid;
                if (k4 < n4) {
                    ss += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
                    const int grp = k4 / NP, pl = k4 - grp * NP;
                    xs[pl * plane_stride + grp] = v[j];
                }
            }
        }
    } else {
        // every thread merges the splits of its own elements: statistics and partials of a batch are all
        // requested before the first is used, so a batch costs one memory round trip
        const int ns = src.nsplit;
        for (int base = 0; base < n4; base += 512) {
            float4 raw[2][MERGE_MAX_SPLIT];
            float ms[2][MERGE_MAX_SPLIT], ls[2][MERGE_MAX_SPLIT];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int kc = min(base + j * 256 + tid, n4 - 1);
                const int h = 4 * kc / src.DH, dim = 4 * kc - h * src.DH;
                const float* pm = src.part_ml + (size_t)h * ns * 2;
                const float* pa = src.part_acc + (size_t)h * ns * src.DH + dim;
#pragma unroll
                for (int s = 0; s < MERGE_MAX_SPLIT; ++s) {
                    const int sc = min(s, ns - 1);
                    ms[j][s] = load_f32(pm + 2 * sc); ls[j][s] = load_f32(pm + 2 * sc + 1);
                    raw[j][s] = as_float4(load16(pa + (size_t)sc * src.DH));
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int k4 = base + j * 256 + tid;
                float M = -INFINITY, L = 0.f;
#pragma unroll
                for (int s = 0; s < MERGE_MAX_SPLIT; ++s) if (s < ns) M = fmaxf(M, ms[j][s]);
                float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int s = 0; s < MERGE_MAX_SPLIT; ++s) {
                    const float w = (s < ns && ms[j][s] > -INFINITY) ? expf(ms[j][s] - M) : 0.f;
                    L += ls[j][s] * w;
                    r.x = fmaf(raw[j][s].x, w, r.x); r.y = fmaf(raw[j][s].y, w, r.y);
                    r.z = fmaf(raw[j][s].z, w, r.z); r.w = fmaf(raw[j][s].w, w, r.w);
                }
                const float inv = 1.f / L;
                if (k4 < n4) {
                    const int grp = k4 / NP, pl = k4 - grp * NP;
                    xs[pl * plane_stride + grp] = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
                }
            }
        }
    }
    if (pad) {
        for (int grp = Kg + tid; grp < KT * 256; grp += 256)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) xs[pl * plane_stride + grp] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (tid < 64)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl) xs[pl * plane_stride + plane_stride - 64 + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// The same staging for a plain vector x (times a gain if GAIN) of at most 1024 NB elements, in two steps with the
// loads held in registers between them.  A caller that requests the vector before its first weight tiles gets it
// back first (loads return in issue order) and stages it while the tiles are still on their way.  Straight-line
// code on purpose: a loop with loads between the tile requests and their uses would make the compiler wait for
// all of them.
template <int NB, bool GAIN>
struct EarlyBatch { float4 v[NB], gn[GAIN ? NB : 1]; };

template <int NB, bool GAIN>
__device__ __forceinline__ void early_request(EarlyBatch<NB, GAIN>& b, const float* x, const float* gain, int K) {
    const int tid = threadIdx.x, n4 = K >> 2;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int k4 = min(j * 256 + tid, n4 - 1);
        b.v[j] = as_float4(load16(x + 4 * (size_t)k4));
        if (GAIN) b.gn[j] = as_float4(load16(gain + 4 * (size_t)k4));
    }
}

// Needs K <= 1024 NB (256 KT - Kg < 256 always holds: one padding group per thread at most).
template <typename WT, int NB, bool GAIN>
__device__ __forceinline__ float early_stage(const EarlyBatch<NB, GAIN>& b, float4* xs, int plane_stride, int K, int Kg, int KT,
                                             float* red) {
    constexpr int NP = Elem<WT>::EPL / 4;
    const int tid = threadIdx.x, n4 = K >> 2;
    const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
    if (Kg + tid < KT * 256)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) xs[pl * plane_stride + Kg + tid] = zero;
    if (tid < 64)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) xs[pl * plane_stride + plane_stride - 64 + tid] = zero;
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int k4 = j * 256 + tid;
        if (k4 < n4) {
            float4 v = b.v[j];
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            if (GAIN) { const float4 gn = b.gn[j]; v = make_float4(v.x * gn.x, v.y * gn.y, v.z * gn.z, v.w * gn.w); }
            const int grp = k4 / NP, pl = k4 - grp * NP;
            xs[pl * plane_stride + grp] = v;
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// ---------------------------------------------------------------------------------------------
// matrix-vector product of one wave over its share of the rows, through a ring of register tiles
// ---------------------------------------------------------------------------------------------

constexpr int RING = 4;

template <typename WT>
struct Phase {
    const WT* W;
    int rows, K, Kg, KT, units, u0, u1;   // this wave owns units [u0, u1)
    int rot;                              // first k-tile of the wave's walk over a unit, see make_phase
};

struct Cursor { int u, kt; };

// One ring slot: a tile of weights (2 rows x 4 k-steps) plus the two values the unit's epilogue needs
// from memory (residual pair, or rotary cos / sin).  They are requested with the tile, because a load
// issued at epilogue time could only be waited for together with every tile load issued before it.
struct Slot {
    uint4 v[8];
    float e0, e1;
};

// The same with the split of the units over the waves given by the host: uq = units / waves, ur = units % waves, the
// first ur waves own one unit more.  No division in the kernel: the two 64-bit divisions of make_phase stand between
// the kernel's start and its first weight request (about a microsecond).
template <typename WT, int EPI>
__device__ __forceinline__ Phase<WT> make_phase_split(const void* W, int rows, int K, int units, int uq, int ur) {
    Phase<WT> p;
    p.W = (const WT*)W; p.rows = rows; p.K = K; p.Kg = K / Elem<WT>::EPL;
    p.KT = (p.Kg + 255) / 256; p.units = units;
    const int gw = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    p.u0 = gw * uq + min(gw, ur); p.u1 = p.u0 + uq + (gw < ur ? 1 : 0);
    p.rot = (int)((unsigned)gw % (unsigned)p.KT);
    return p;
}

template <typename WT, int EPI>
__device__ __forceinline__ Phase<WT> make_phase(const void* W, int rows, int K, int units) {
    Phase<WT> p;
    p.W = (const WT*)W; p.rows = rows; p.K = K; p.Kg = K / Elem<WT>::EPL;
    p.KT = (p.Kg + 255) / 256; p.units = units;
    const long long gw = (long long)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), tw = (long long)gridDim.x * 4;
    p.u0 = (int)(units * gw / tw); p.u1 = (int)(units * (gw + 1) / tw);
    // Every wave walks the k-tiles of its units in rotated order from a tile of its own: waves that all read the same
    // columns of their rows at the same time (the rows lie a multiple of the row length apart) load the memory channels
    // unevenly (measured: 2 % of the decoding step at d_model 8192, 0.3 % at 4096).
    p.rot = (int)(gw % p.KT);
    return p;
}

__device__ __forceinline__ void advance(Cursor& c, int KT) {
    if (++c.kt == KT) { c.kt = 0; ++c.u; }
}

// Requests tile (c.u, c.kt): rows (rA, rB) of the unit, k-steps 4 kt .. 4 kt + 3.  Past the end of the
// wave's range the last tile is requested again (a cache hit); addresses always stay inside W.
template <typename WT, int EPI>
__device__ __forceinline__ void tile_load_w(Slot& sl, const Phase<WT>& p, const Cursor& c, int lane, const Geom& g) {
    uint4 (&v)[8] = sl.v;
    constexpr int EPL = Elem<WT>::EPL;
    const bool past = c.u >= p.u1;
    const int u = past ? max(min(p.u1, p.units) - 1, 0) : c.u;
    int kt = (past ? p.KT - 1 : c.kt) + p.rot;
    kt = kt >= p.KT ? kt - p.KT : kt;
    int rA, rB;
    unit_rows<EPI>(u, p.rows, g, rA, rB);
    const WT* pa = p.W + (size_t)rA * p.K;
    const WT* pb = p.W + (size_t)rB * p.K;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int gi = min((kt * 4 + s) * 64 + lane, p.Kg - 1);
        v[2 * s] = load16_stream(pa + (size_t)gi * EPL);
        v[2 * s + 1] = load16_stream(pb + (size_t)gi * EPL);
    }
}

// The epilogue operands of the same tile's unit.
template <typename WT, int EPI>
__device__ __forceinline__ void tile_load_e(Slot& sl, const Phase<WT>& p, const Cursor& c, const Geom& g, const EpiOut& eo) {
    const bool past = c.u >= p.u1;
    const int u = past ? max(min(p.u1, p.units) - 1, 0) : c.u;
    int rA, rB;
    unit_rows<EPI>(u, p.rows, g, rA, rB);
    if (EPI == EPI_RESID) {
        sl.e0 = load_f32(eo.res + rA); sl.e1 = load_f32(eo.res + rB);
    } else if (EPI == EPI_QKV) {
        const int hs = g.dh == 128 ? 6 : 5, h = u >> hs, i = u & ((1 << hs) - 1);
        const size_t ri = ((size_t)eo.pos << hs) + i;
        // as loaded: a select here would have to wait for the loads (finish_unit drops them for value rows)
        sl.e0 = load_f32(eo.rope_cos + ri); sl.e1 = load_f32(eo.rope_sin + ri);
    } else { sl.e0 = 0.f; sl.e1 = 0.f; }
}

template <typename WT, int EPI>
__device__ __forceinline__ void tile_load(Slot& sl, const Phase<WT>& p, const Cursor& c, int lane, const Geom& g, const EpiOut& eo) {
    tile_load_w<WT, EPI>(sl, p, c, lane, g);
    tile_load_e<WT, EPI>(sl, p, c, g, eo);
}

// Epilogue of unit u, by one lane: sa, sb are the finished dot products, e0 / e1 the slot's operands.
template <typename WT, int EPI>
__device__ __forceinline__ void finish_unit(int u, float sa, float sb, float e0, float e1, const EpiOut& o, const Geom& g) {
    if (EPI == EPI_STORE) {
        o.y[2 * u] = sa;
        if (2 * u + 1 < o.rows) o.y[2 * u + 1] = sb;
    } else if (EPI == EPI_RESID) {
        // vectors that the next kernel of the step reads are written through (it may already be running)
        store_coherent(o.y + 2 * u, e0 + sa);
        if (2 * u + 1 < o.rows) store_coherent(o.y + 2 * u + 1, e1 + sb);
    } else if (EPI == EPI_SWIGLU) {
        store_coherent(o.y + u, sa / (1.f + expf(-sa)) * sb);
    } else {
        const int hs = g.dh == 128 ? 6 : 5, half = 1 << hs;
        const int h = u >> hs, i = u & (half - 1);
        if (h >= g.Hq + g.Hkv) { e0 = 1.f; e1 = 0.f; }                 // value rows are not rotated
        const float ra = sa * e0 - sb * e1, rb = sb * e0 + sa * e1;
        const size_t seq_off = (size_t)o.seq * g.kv_seq_stride;
        if (h < g.Hq) { store_coherent(o.q_out + h * g.dh + i, ra); store_coherent(o.q_out + h * g.dh + i + half, rb); }
        else if (h < g.Hq + g.Hkv) {
            WT* kp = (WT*)o.kv_layer + seq_off + (size_t)(h - g.Hq) * g.kv_head_stride + (size_t)o.pos * g.dh;
            kv_store(kp + i, ra, g.kv_lo_offset); kv_store(kp + i + half, rb, g.kv_lo_offset);
        } else {
            const size_t head_off = seq_off + (size_t)(h - g.Hq - g.Hkv) * g.kv_head_stride;
            if (g.kv_v_offset) {
                WT* vp = (WT*)o.kv_layer + g.kv_v_offset + head_off + (size_t)o.pos * g.dh;
                kv_store(vp + i, ra, g.kv_lo_offset); kv_store(vp + i + half, rb, g.kv_lo_offset);
            }
            if (g.kv_vt_offset) {
                WT* vt = (WT*)o.kv_layer + g.kv_vt_offset + head_off;
                kv_store(vt + vt_tile_off(o.pos, i), ra, g.kv_lo_offset);
                kv_store(vt + vt_tile_off(o.pos, i + half), rb, g.kv_lo_offset);
            }
        }
    }
}

// Multiplies one tile with the staged vector.  xs: planar LDS copy of x (plane p holds elements
// 4p..4p+3 of every group of EPL), zero beyond Kg; tiles past the end read a block of zeros.
template <typename WT>
__device__ __forceinline__ void tile_fma(const uint4 (&v)[8], const float4* xs, int plane_stride, int zero_group,
                                         bool past, int kt, int lane, float& accA, float& accB) {
    constexpr int EPL = Elem<WT>::EPL;
    constexpr int NP = EPL / 4;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int gi = past ? zero_group + lane : (kt * 4 + s) * 64 + lane;
        float xv[EPL], wa[EPL], wb[EPL];
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) {
            const float4 t = xs[pl * plane_stride + gi];
            xv[4 * pl] = t.x; xv[4 * pl + 1] = t.y; xv[4 * pl + 2] = t.z; xv[4 * pl + 3] = t.w;
        }
        Elem<WT>::expand(v[2 * s], wa);
        Elem<WT>::expand(v[2 * s + 1], wb);
#pragma unroll
        for (int e = 0; e < EPL; ++e) { accA = fmaf(wa[e], xv[e], accA); accB = fmaf(wb[e], xv[e], accB); }
    }
}

// First RING tiles of a phase; issued before the grid barrier that precedes the phase.
template <typename WT, int EPI>
__device__ __forceinline__ void phase_prefetch(Slot (&ring)[RING], const Phase<WT>& p, Cursor& lc, int lane, const Geom& g,
                                               const EpiOut& eo) {
    lc.u = p.u0; lc.kt = 0;
#pragma unroll
    for (int j = 0; j < RING; ++j) {
        tile_load<WT, EPI>(ring[j], p, lc, lane, g, eo);
        advance(lc, p.KT);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// The same in two steps, for callers that learn the epilogue operands' addresses (the position) only after
// the weight requests are out.
template <typename WT, int EPI>
__device__ __forceinline__ void phase_prefetch_w(Slot (&ring)[RING], const Phase<WT>& p, int lane, const Geom& g) {
    Cursor c; c.u = p.u0; c.kt = 0;
#pragma unroll
    for (int j = 0; j < RING; ++j) {
        tile_load_w<WT, EPI>(ring[j], p, c, lane, g);
        advance(c, p.KT);
        __builtin_amdgcn_sched_barrier(0);      // tile by tile: the first tile's loads are the first to return
    }
}
template <typename WT, int EPI>
__device__ __forceinline__ void phase_prefetch_e(Slot (&ring)[RING], const Phase<WT>& p, Cursor& lc, const Geom& g, const EpiOut& eo) {
    lc.u = p.u0; lc.kt = 0;
#pragma unroll
    for (int j = 0; j < RING; ++j) {
        tile_load_e<WT, EPI>(ring[j], p, lc, g, eo);
        advance(lc, p.KT);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// Runs a phase whose first RING tiles are already in `ring`.  The loop only parks each finished unit
// (two dot products and the slot's epilogue operands) in the wave's LDS area `done`; the epilogues, with
// their global stores, run after the loop, one unit per lane.  Keeping every global memory instruction
// of the loop unconditional lets the compiler count the outstanding loads exactly, so a tile is waited
// for while the three younger ones stay in flight.
// best_v / best_i: argmax of the stored values (EPI_STORE only), valid in every lane afterwards.
template <typename WT, int EPI>
__device__ __forceinline__ void phase_run(Slot (&ring)[RING], const Phase<WT>& p, Cursor& lc, const float4* xs,
                                          int plane_stride, float nscale, const EpiOut& eo, const Geom& g, int lane,
                                          float4* done, float& best_v, int& best_i) {
    const int zero_group = plane_stride - 64;
    const int T = (p.u1 - p.u0) * p.KT;
    Cursor cc; cc.u = p.u0; cc.kt = 0;
    float accA = 0.f, accB = 0.f;
    for (int t = 0; t < T; t += RING) {
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            const bool past = cc.u >= p.u1;
            const int ktp = cc.kt + p.rot >= p.KT ? cc.kt + p.rot - p.KT : cc.kt + p.rot;      // the tile that was requested
            tile_fma<WT>(ring[j].v, xs, plane_stride, zero_group, past, ktp, lane, accA, accB);
            // The slot's epilogue operands are parked before the slot is requested again: read after the request
            // they would have to be copied aside when the loop rotates, and the copy waits for every load in flight.
            if (!past && cc.kt == p.KT - 1) {
                const float sa = wave_sum(accA) * nscale, sb = wave_sum(accB) * nscale;
                if (lane == 0) done[cc.u - p.u0] = make_float4(sa, sb, ring[j].e0, ring[j].e1);
                accA = 0.f; accB = 0.f;
            }
            __builtin_amdgcn_sched_barrier(0);
            tile_load<WT, EPI>(ring[j], p, lc, lane, g, eo);
            advance(lc, p.KT);
            __builtin_amdgcn_sched_barrier(0);
            advance(cc, p.KT);
        }
    }
    for (int ul = lane; ul < p.u1 - p.u0; ul += 64) {
        const float4 r = done[ul];          // written by lane 0 of this same wave
        const int u = p.u0 + ul;
        finish_unit<WT, EPI>(u, r.x, r.y, r.z, r.w, eo, g);
        if (EPI == EPI_STORE) {
            amax_merge(best_v, best_i, r.x, 2 * u);
            if (2 * u + 1 < p.rows) amax_merge(best_v, best_i, r.y, 2 * u + 1);
        }
    }
    if (EPI == EPI_STORE) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(best_v, o, 64); const int oi = __shfl_xor(best_i, o, 64);
            amax_merge(best_v, best_i, ov, oi);
        }
    }
}

}  // namespace asynclm
