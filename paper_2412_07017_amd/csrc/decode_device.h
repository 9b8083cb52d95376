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
__device__ __forceinline__ void kv_store(float* p, float v, size_t) { *p = v; }
__device__ __forceinline__ void kv_store(bf16_t* p, float v, size_t lo_offset) {
    const bf16_t hi = f32_to_bf16(v);
    *p = hi;
    if (lo_offset) p[lo_offset] = f32_to_bf16(v - __uint_as_float((uint32_t)hi << 16));
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

// Called by one lane with the two finished dot products of unit u.
template <typename WT, int EPI>
__device__ __forceinline__ void gemv_finish(int u, float sa, float sb, const EpiOut& o, const Geom& g) {
    if (EPI == EPI_STORE) {
        o.y[2 * u] = sa;
        if (2 * u + 1 < o.rows) o.y[2 * u + 1] = sb;
    } else if (EPI == EPI_RESID) {
        o.y[2 * u] = o.res[2 * u] + sa;
        if (2 * u + 1 < o.rows) o.y[2 * u + 1] = o.res[2 * u + 1] + sb;
    } else if (EPI == EPI_SWIGLU) {
        o.y[u] = sa / (1.f + expf(-sa)) * sb;
    } else {
        const int hs = g.dh == 128 ? 6 : 5, half = 1 << hs;
        const int h = u >> hs, i = u & (half - 1);
        const int pos = o.pos;
        const size_t seq_off = (size_t)o.seq * g.kv_seq_stride;
        if (h < g.Hq + g.Hkv) {
            const float c = o.rope_cos[(size_t)pos * half + i], s = o.rope_sin[(size_t)pos * half + i];
            const float ra = sa * c - sb * s, rb = sb * c + sa * s;
            if (h < g.Hq) { o.q_out[h * g.dh + i] = ra; o.q_out[h * g.dh + i + half] = rb; }
            else {
                WT* kp = (WT*)o.kv_layer + seq_off + (size_t)(h - g.Hq) * g.kv_head_stride + (size_t)pos * g.dh;
                kv_store(kp + i, ra, g.kv_lo_offset); kv_store(kp + i + half, rb, g.kv_lo_offset);
            }
        } else {
            const size_t head_off = seq_off + (size_t)(h - g.Hq - g.Hkv) * g.kv_head_stride;
            WT* vp = (WT*)o.kv_layer + g.kv_v_offset + head_off + (size_t)pos * g.dh;
            kv_store(vp + i, sa, g.kv_lo_offset); kv_store(vp + i + half, sb, g.kv_lo_offset);
            if (g.kv_vt_offset) {   // transposed copy [dh][max_pos] read by the append-chunk attention
                WT* vt = (WT*)o.kv_layer + g.kv_vt_offset + head_off + pos;
                kv_store(vt + (size_t)i * g.max_pos, sa, g.kv_lo_offset);
                kv_store(vt + (size_t)(i + half) * g.max_pos, sb, g.kv_lo_offset);
            }
        }
    }
}

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
template <typename WT>
__device__ __forceinline__ float stage_vector(float4* xs, int plane_stride, const VecSource& src, int K, int Kg, int KT,
                                              bool pad, float* red) {
    constexpr int NP = Elem<WT>::EPL / 4;
    const int tid = threadIdx.x, n4 = K >> 2;
    float ss = 0.f;
    if (src.x) {
        for (int base = 0; base < n4; base += 1024) {
            float4 v[4], gn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k4 = min(base + j * 256 + tid, n4 - 1);
                v[j] = as_float4(load16(src.x + 4 * (size_t)k4));
                gn[j] = src.gain ? as_float4(load16(src.gain + 4 * (size_t)k4)) : make_float4(1.f, 1.f, 1.f, 1.f);
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

}  // namespace asynclm
