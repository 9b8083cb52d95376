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

// LDS of one attention workgroup
template <int DH, int G>
struct AttnSmem {
    float m[4][G], l[4][G], acc[4][G][DH];
};

// Positions [s0, s1) of one kv head for its G query heads, by one workgroup of 4 waves.
// q: [Hq*DH] rotated, unscaled.  Kp / Vp: row-major planes of this kv head (row = position).
// After the call (it ends with a __syncthreads) sm.m / sm.l / sm.acc hold the per-wave online-softmax
// state; attn_fold turns them into the workgroup's (M, L, A[dim]).
template <typename KVT, int DH, int G, bool PAIR, int UN = 4>
__device__ __forceinline__ void attn_partial(const float* __restrict__ q, const KVT* __restrict__ Kp,
                                             const KVT* __restrict__ Vp, size_t lo_offset, int kvh, int s0, int s1,
                                             float scale, AttnSmem<DH, G>& sm) {
    constexpr int EPL = Elem<KVT>::EPL;
    constexpr int LPR = DH / EPL;       // lanes that cover one cached row
    constexpr int PPW = 64 / LPR;       // positions per wave-wide load
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, c = lane % LPR;

    float qr[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) qr[h][e] = q[(kvh * G + h) * DH + c * EPL + e] * scale;

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[h][e] = 0.f;
    }

    // UN position groups per trip: all their K/V loads are issued before the first is used
    for (int p0 = s0 + wave * PPW; p0 < s1; p0 += 4 * PPW * UN) {
        uint4 kr[UN], vr[UN], krl[PAIR ? UN : 1], vrl[PAIR ? UN : 1];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int p = p0 + u * 4 * PPW + sub;
            const int pc = p < s1 ? p : s1 - 1;
            kr[u] = load16(Kp + (size_t)pc * DH + c * EPL);
            vr[u] = load16(Vp + (size_t)pc * DH + c * EPL);
            if (PAIR) {
                krl[u] = load16(Kp + lo_offset + (size_t)pc * DH + c * EPL);
                vrl[u] = load16(Vp + lo_offset + (size_t)pc * DH + c * EPL);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const bool valid = p0 + u * 4 * PPW + sub < s1;
            float kf[EPL], vf[EPL];
            Elem<KVT>::expand(kr[u], kf);
            Elem<KVT>::expand(vr[u], vf);
            if (PAIR) {
                float kl[EPL], vl[EPL];
                Elem<KVT>::expand(krl[u], kl);
                Elem<KVT>::expand(vrl[u], vl);
#pragma unroll
                for (int e = 0; e < EPL; ++e) { kf[e] += kl[e]; vf[e] += vl[e]; }
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) s = fmaf(qr[h][e], kf[e], s);
#pragma unroll
                for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o, 64);
                if (!valid) s = -INFINITY;
                float mx = s;
#pragma unroll
                for (int o = LPR; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
                // group u = 0 always holds the valid position p0, so m is finite from then on
                const float mn = fmaxf(m[h], mx);
                const float corr = expf(m[h] - mn);     // exp(-inf) = 0 on the very first group
                const float pr = expf(s - mn);
                l[h] = l[h] * corr + pr;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[h][e] = fmaf(pr, vf[e], acc[h][e] * corr);
                m[h] = mn;
            }
        }
    }

    // fold the PPW position groups of the wave (they share m)
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) {
            l[h] += __shfl_xor(l[h], o, 64);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[h][e] += __shfl_xor(acc[h][e], o, 64);
        }
        if (sub == 0) {
            if (c == 0) { sm.m[wave][h] = m[h]; sm.l[wave][h] = l[h]; }
#pragma unroll
            for (int e = 0; e < EPL; ++e) sm.acc[wave][h][c * EPL + e] = acc[h][e];
        }
    }
    __syncthreads();
}

// Fold the four waves for (query head h of the group, channel dim); a wave without positions has m = -inf.
template <int DH, int G>
__device__ __forceinline__ void attn_fold(const AttnSmem<DH, G>& sm, int h, int dim, float& M, float& L, float& A) {
    M = fmaxf(fmaxf(sm.m[0][h], sm.m[1][h]), fmaxf(sm.m[2][h], sm.m[3][h]));
    L = 0.f; A = 0.f;
    if (M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = expf(sm.m[w][h] - M);
            L += sm.l[w][h] * f; A += sm.acc[w][h][dim] * f;
        }
    }
}

}  // namespace asynclm
