// Append-chunk path on gfx950 (bf16 models): M = 2..CHUNK_MAX rows per forward pass, used by
// interrupt injection and prefill.  Weights are streamed from HBM once per pass; every linear
// map and the causal chunk attention run on the matrix cores (v_mfma_f32_32x32x16_bf16), with
// fp32 accumulation.  Activations are carried as a pair of bf16 planes, hi = bf16(x) and
// lo = bf16(x - hi), and each product is formed as W*hi + W*lo, so the chunk path keeps about
// 16 mantissa bits like the fp32 activations of the single-row path.
//
// Matrix-core operand layout used throughout (wave of 64 lanes, lane = 32 g + i):
//   A[32 x 16]: lane (i, g) holds A[i][8g .. 8g+7]        (8 bf16 = one 16-byte register quad)
//   B[16 x 32]: lane (j, g) holds B[8g .. 8g+7][j]
//   D[32 x 32]: lane (j, g) holds D[8b + 4g + r][j] in register 4b + r  (b, r = 0..3)
// Within a k-block of 128 elements, MFMA step t, lane half g, element e is k = 16 t + 8 g + e.
//
// Memory access.  A wave-wide 16-byte load is cheap when its 64 lanes cover few cache lines, so:
//  * activations (the B operand) are kept in global memory in operand order ("tiled planes"):
//    element (row m, column k) lives at ((((m/32 * K/128 + k/128) * 8 + t) * 2 + g) * 32 + m%32) * 8 + e,
//    and the 64 lanes of a B load read one contiguous KiB;
//  * weights (the A operand, row-major in HBM) are loaded 4 rows x 256 contiguous bytes per
//    instruction and transposed into operand order through a wave-private, XOR-swizzled LDS tile.
// In the chunk attention, which is small next to the weight streaming, every lane instead reads 128
// contiguous bytes of its own K / V^T row (k = 64 g + 8 t + e there).
#include "common.h"
#include "launch.h"

namespace asynclm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16 mfma_bf16(const uint4& a, const uint4& b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
    hi = f32_to_bf16(v);
    lo = f32_to_bf16(v - __uint_as_float((uint32_t)hi << 16));
}

// offset (elements) of (row m, column k) in a tiled plane with K columns
__device__ __forceinline__ size_t tiled_off(int m, int k, int K) {
    const int kk = k & 127;
    return ((((size_t)(m >> 5) * (K >> 7) + (k >> 7)) * 8 + (kk >> 4)) * 2 + ((kk >> 3) & 1)) * 256 + (size_t)(m & 31) * 8 + (kk & 7);
}

// ---------------------------------------------------------------------------------------------
// bookkeeping and small row-wise kernels
// ---------------------------------------------------------------------------------------------

// Resolves the tokens that are chosen on the device (first row of a group), records them, moves the
// sequence lengths, and fills the step descriptor that the single-row head kernels read.
__global__ void k_begin_chunk(ChunkTable* tab, StepDesc* step, SeqState* st, int32_t* chosen) {
    const int ng = tab->ngroups;
    for (int gi = threadIdx.x; gi < ng; gi += blockDim.x) {
        const ChunkGroup G = tab->group[gi];
        if (G.forced != -2) {
            const int32_t tok = G.forced >= 0 ? G.forced : st[G.seq].next_token;
            tab->row[G.row0].token = tok;
            chosen[gi] = tok;
        }
        st[G.seq].len = G.pos0 + G.n;
    }
    if (threadIdx.x == 0) {
        step->token = -1; step->pos = tab->group[0].pos0; step->seq = tab->group[0].seq; step->rows = tab->rows;
    }
}

// x[m][:] = E[token_m][:]   (one workgroup per row)
__global__ __launch_bounds__(256) void k_chunk_embed(const bf16_t* __restrict__ E, const ChunkTable* __restrict__ tab,
                                                     float* __restrict__ x, int d) {
    const int m = blockIdx.x;
    const bf16_t* row = E + (size_t)tab->row[m].token * d;
    for (int i = threadIdx.x; i < d; i += 256) x[(size_t)m * d + i] = Elem<bf16_t>::load1(row + i);
}

constexpr int ROW_VEC_MAX = 8;      // float4 groups per thread of a row kernel: d <= 8192

// One row by one workgroup: v = x[m] + sum_s P[s][row pm] (S <= CHUNK_GEMM_MAX_SPLIT planes; all loads of the
// row are issued before the first use, the gain's of the following norm among them), returns the sum of squares
// over the workgroup.  Thread tid owns the float4 groups tid + 256 u.
__device__ __forceinline__ float row_gather(const float* __restrict__ xr, const float* __restrict__ Pr, int S,
                                            size_t s_stride, int d4, int tid, const float* __restrict__ gain,
                                            float4 (&v)[ROW_VEC_MAX], float4 (&gn)[ROW_VEC_MAX], float* red) {
    const float4* x4 = reinterpret_cast<const float4*>(xr);
    float ss = 0.f;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        constexpr int HU = ROW_VEC_MAX / 2;
        if (hf * HU * 256 < d4) {                               // uniform: the upper half only for d > 4096
            float4 p[HU][CHUNK_GEMM_MAX_SPLIT];
#pragma unroll
            for (int u = 0; u < HU; ++u) {
                const int i4 = min(tid + 256 * (hf * HU + u), d4 - 1);      // past the end: a repeated load, dropped below
                v[hf * HU + u] = x4[i4];
                gn[hf * HU + u] = reinterpret_cast<const float4*>(gain)[i4];
#pragma unroll
                for (int s = 0; s < CHUNK_GEMM_MAX_SPLIT; ++s)
                    p[u][s] = Pr ? reinterpret_cast<const float4*>(Pr + (size_t)min(s, S - 1) * s_stride)[i4] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < HU; ++u) {
                float4& w = v[hf * HU + u];
#pragma unroll
                for (int s = 0; s < CHUNK_GEMM_MAX_SPLIT; ++s) {
                    const float k = s < S ? 1.f : 0.f;
                    w.x += k * p[u][s].x; w.y += k * p[u][s].y; w.z += k * p[u][s].z; w.w += k * p[u][s].w;
                }
                if (tid + 256 * (hf * HU + u) < d4) ss += w.x * w.x + w.y * w.y + w.z * w.z + w.w * w.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < HU; ++u) { v[hf * HU + u] = make_float4(0.f, 0.f, 0.f, 0.f); gn[hf * HU + u] = v[hf * HU + u]; }
        }
    }
    ss = wave_sum(ss);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// v * sc * gain -> tiled bf16 hi/lo planes at row `mo`
__device__ __forceinline__ void row_emit(const float4 (&v)[ROW_VEC_MAX], float sc, const float4 (&gain)[ROW_VEC_MAX], int d,
                                         int tid, int mo, bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo) {
    const int d4 = d >> 2;
#pragma unroll
    for (int u = 0; u < ROW_VEC_MAX; ++u) {
        const int i4 = tid + 256 * u;
        if (i4 < d4) {
            const float4 gn = gain[u];
            bf16_t h0, l0, h1, l1, h2, l2, h3, l3;
            split_bf16(v[u].x * sc * gn.x, h0, l0); split_bf16(v[u].y * sc * gn.y, h1, l1);
            split_bf16(v[u].z * sc * gn.z, h2, l2); split_bf16(v[u].w * sc * gn.w, h3, l3);
            const size_t o = tiled_off(mo, 4 * i4, d);       // 4 consecutive columns stay inside one 8-element group
            *reinterpret_cast<uint2*>(out_hi + o) = make_uint2(h0 | ((uint32_t)h1 << 16), h2 | ((uint32_t)h3 << 16));
            *reinterpret_cast<uint2*>(out_lo + o) = make_uint2(l0 | ((uint32_t)l1 << 16), l2 | ((uint32_t)l3 << 16));
        }
    }
}

// x[m] += sum_s P[s][m]  (if P), then RMSNorm with `gain` -> tiled bf16 hi/lo planes.
// One workgroup per row; P has row stride n_stride and split stride s_stride (elements).
__global__ __launch_bounds__(256) void k_chunk_resid_norm(float* __restrict__ x, const float* __restrict__ P, int S,
                                                          size_t s_stride, int n_stride, const float* __restrict__ gain,
                                                          float eps, int d, bf16_t* __restrict__ out_hi,
                                                          bf16_t* __restrict__ out_lo) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x, d4 = d >> 2;
    float* xr = x + (size_t)m * d;
    float4 v[ROW_VEC_MAX], gn[ROW_VEC_MAX];
    const float ss = row_gather(xr, P ? P + (size_t)m * n_stride : nullptr, S, s_stride, d4, tid, gain, v, gn, red);
    if (P) {
#pragma unroll
        for (int u = 0; u < ROW_VEC_MAX; ++u)
            if (tid + 256 * u < d4) reinterpret_cast<float4*>(xr)[tid + 256 * u] = v[u];
    }
    row_emit(v, rsqrtf(ss / (float)d + eps), gn, d, tid, m, out_hi, out_lo);
}

// Last row of group `group` only: out[:] = x[row] + sum_s P[s][row]  (residual stream handed to the
// single-row output head); the step descriptor gets the group's sequence.
__global__ __launch_bounds__(256) void k_chunk_last_row(const float* __restrict__ x, const float* __restrict__ P, int S,
                                                        size_t s_stride, int n_stride, int d, const ChunkTable* __restrict__ tab,
                                                        int group, StepDesc* step, float* __restrict__ out) {
    const ChunkGroup G = tab->group[group];
    const int row = G.row0 + G.n - 1;
    if (blockIdx.x == 0 && threadIdx.x == 0) step->seq = G.seq;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d; i += gridDim.x * 256) {
        float v = x[(size_t)row * d + i];
        for (int s = 0; s < S; ++s) v += P[s * s_stride + (size_t)row * n_stride + i];
        out[i] = v;
    }
}

// Workgroup = group: if the group wants logits, its last row (residual + down-projection partials), normalised
// with the final gain, becomes row `head` of the tiled planes that feed the output-head product.
__global__ __launch_bounds__(256) void k_chunk_head_rows(const float* __restrict__ x, const float* __restrict__ P, int S,
                                                         size_t s_stride, int n_stride, const float* __restrict__ gain,
                                                         float eps, int d, const ChunkTable* __restrict__ tab,
                                                         bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo) {
    __shared__ float red[4];
    const ChunkGroup G = tab->group[blockIdx.x];
    if (G.head < 0) return;
    const int row = G.row0 + G.n - 1, tid = threadIdx.x, d4 = d >> 2;
    float4 v[ROW_VEC_MAX], gn[ROW_VEC_MAX];
    const float ss = row_gather(x + (size_t)row * d, P + (size_t)row * n_stride, S, s_stride, d4, tid, gain, v, gn, red);
    row_emit(v, rsqrtf(ss / (float)d + eps), gn, d, tid, G.head, out_hi, out_lo);
}

// Workgroup = group that wants logits: row `head` of the output-head product -> logits of its sequence,
// greedy argmax (lowest index on ties) -> next_token.
__global__ __launch_bounds__(1024) void k_chunk_logits(const float* __restrict__ P, int V, const ChunkTable* __restrict__ tab,
                                                       float* __restrict__ logits_base, SeqState* st,
                                                       const int32_t* __restrict__ banned) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const ChunkGroup G = tab->group[blockIdx.x];
    if (G.head < 0) return;
    const float* src = P + (size_t)G.head * V;
    float* dst = logits_base + (size_t)G.seq * V;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float bv = -INFINITY; int bi = 0x7fffffff;
    const int32_t* ban = banned + (size_t)G.seq * (1 + BAN_MAX);
    const int nban = ban[0];
    for (int i = tid; i < V; i += 1024) {
        const float v = src[i];
        dst[i] = v;
        bool allowed = true;
        for (int k = 0; k < nban; ++k) allowed = allowed && i != ban[1 + k];
        if (allowed && v > bv) { bv = v; bi = i; }  // i ascends: the first maximum is kept
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; ++w)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        st[G.seq].next_token = bi;
    }
}

// a[m][f] = silu(sum_s gate) * (sum_s up) -> tiled hi/lo planes
__global__ __launch_bounds__(256) void k_chunk_swiglu(const float* __restrict__ P, int S, size_t s_stride, int n_stride,
                                                      int F, bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo) {
    const int m = blockIdx.y;
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= F) return;
    float gt = 0.f, up = 0.f;
    for (int s = 0; s < S; ++s) {
        const float* p = P + s * s_stride + (size_t)m * n_stride;
        gt += p[f]; up += p[F + f];
    }
    bf16_t hi, lo;
    split_bf16(gt / (1.f + expf(-gt)) * up, hi, lo);
    const size_t o = tiled_off(m, f, F);
    out_hi[o] = hi; out_lo[o] = lo;
}

// Rotary embedding of q and k, K/V cache write (row-major planes and the transposed V planes), scaled q
// as hi/lo planes [Hkv][q_cols][dh] with the columns of a group ordered [q head in the kv group][row].
// grid (heads = Hq + 2 Hkv, rows), dh/2 threads.
__global__ void k_chunk_rope_kv(const float* __restrict__ P, int S, size_t s_stride, int n_stride, Geom g,
                                const ChunkTable* __restrict__ tab, const float* __restrict__ rope_cos,
                                const float* __restrict__ rope_sin, bf16_t* __restrict__ kv_layer,
                                bf16_t* __restrict__ q_hi, bf16_t* __restrict__ q_lo, int q_cols) {
    const int h = blockIdx.x, m = blockIdx.y, i = threadIdx.x, half = g.dh >> 1;
    const ChunkRow R = tab->row[m];
    const int pos = R.pos;
    const size_t seq_off = (size_t)R.seq * g.kv_seq_stride;
    // all partial products and the rotation of this thread in one round of loads, added in split order
    float pa[CHUNK_GEMM_MAX_SPLIT], pb[CHUNK_GEMM_MAX_SPLIT];
#pragma unroll
    for (int s = 0; s < CHUNK_GEMM_MAX_SPLIT; ++s) {
        const float* p = P + (size_t)min(s, S - 1) * s_stride + (size_t)m * n_stride + h * g.dh;
        pa[s] = p[i]; pb[s] = p[i + half];
    }
    const float c = rope_cos[(size_t)pos * half + i], sn = rope_sin[(size_t)pos * half + i];
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int s = 0; s < CHUNK_GEMM_MAX_SPLIT; ++s)
        if (s < S) { a += pa[s]; b += pb[s]; }
    if (h < g.Hq + g.Hkv) {
        const float ra = a * c - b * sn, rb = b * c + a * sn;
        a = ra; b = rb;
    }
    bf16_t ahi, alo, bhi, blo;
    if (h < g.Hq) {
        split_bf16(a * g.scale, ahi, alo); split_bf16(b * g.scale, bhi, blo);
        const int G = g.Hq / g.Hkv, kvh = h / G, gq = h - kvh * G;
        const size_t o = ((size_t)kvh * q_cols + (size_t)G * R.row0 + (size_t)gq * R.n + (m - R.row0)) * g.dh;
        q_hi[o + i] = ahi; q_lo[o + i] = alo; q_hi[o + i + half] = bhi; q_lo[o + i + half] = blo;
        return;
    }
    split_bf16(a, ahi, alo); split_bf16(b, bhi, blo);
    if (h < g.Hq + g.Hkv) {
        bf16_t* kp = kv_layer + seq_off + (size_t)(h - g.Hq) * g.kv_head_stride + (size_t)pos * g.dh;
        kp[i] = ahi; kp[i + half] = bhi; kp[g.kv_lo_offset + i] = alo; kp[g.kv_lo_offset + i + half] = blo;
    } else {
        const int vh = h - g.Hq - g.Hkv;
        if (g.kv_v_offset) {       // row-major values are only kept for the single-row attention kernel
            bf16_t* vp = kv_layer + g.kv_v_offset + seq_off + (size_t)vh * g.kv_head_stride + (size_t)pos * g.dh;
            vp[i] = ahi; vp[i + half] = bhi; vp[g.kv_lo_offset + i] = alo; vp[g.kv_lo_offset + i + half] = blo;
        }
        bf16_t* vt = kv_layer + g.kv_vt_offset + seq_off + (size_t)vh * g.kv_head_stride;
        const size_t oa = vt_tile_off(pos, i), ob = vt_tile_off(pos, i + half);
        vt[oa] = ahi; vt[ob] = bhi; vt[g.kv_lo_offset + oa] = alo; vt[g.kv_lo_offset + ob] = blo;
    }
}

// ---------------------------------------------------------------------------------------------
// skinny GEMM on the matrix cores:  P[s][m][n] = sum_{k in slice s} X[m][k] W[n][k]
// ---------------------------------------------------------------------------------------------
// Which kernel takes a pass (launch_chunk_gemm): up to 32 rows this one (bound by the weight stream, a wave per 32
// weight rows); 33-64 rows k_chunk_gemm_ks (the waves split the k-steps); 65-128 rows k_chunk_gemm_wide with a wave
// per row tile; more rows k_chunk_gemm_wide with 256-row workgroups.  The template serves any MT <= 3; MT = 1 is used.
// Workgroup = 4 waves on 128 weight rows (32 per wave) and one contiguous run of 128-element k-blocks
// (the S workgroups of a row tile split K and write separate partial planes that the consumer adds in
// a fixed order: no atomics, results are bit-reproducible).
//  * weights stream from HBM through a register ring of GemmRing<MT>::N tiles per wave (one tile = the wave's
//    32 rows x 128 columns, loaded 4 rows x 256 contiguous bytes per instruction), are transposed into
//    operand order through a wave-private XOR-swizzled LDS tile and multiplied;
//  * the activations of a k-block (all rows, hi and lo planes: MT x 16 KiB) are shared by the four waves
//    through a double-buffered LDS tile that the workgroup fills one block ahead.
// The loop body has no conditional code around loads or their uses: the prefetches past the end of a run
// re-read its last block (cache hits).  The compiler sinks loads into conditional users
// and then waits for each load right before its product; the scheduling barriers keep the instruction
// scheduler from doing the same within the straight-line body.

// weight tiles per wave in the register ring: four for one row tile, three beyond (registers)
template <int MT> struct GemmRing { static constexpr int N = MT == 1 ? 4 : 3; };

template <int MT>
struct BStage { uint4 v[MT][4]; };

__device__ __forceinline__ void gemm_a_load(uint4 (&a)[8], const bf16_t* wlane, size_t wstep, int blk) {
#pragma unroll
    for (int q = 0; q < 8; ++q) a[q] = load16_stream(wlane + (size_t)blk * 128 + q * wstep);
}

// The same tile from eight rows of the lane's own choice (row q of the lane = tile row 4 q + lane / 16).
__device__ __forceinline__ void gemm_a_load(uint4 (&a)[8], const bf16_t* const (&wrow)[8], int blk) {
#pragma unroll
    for (int q = 0; q < 8; ++q) a[q] = load16_stream(wrow[q] + (size_t)blk * 128);
}

// thread tid stages chunks tid and tid + 256 of the 512 16-byte chunks of each 8 KiB plane tile
template <int MT>
__device__ __forceinline__ void gemm_b_load(BStage<MT>& st, const bf16_t* xh, const bf16_t* xl, int nblk, int blk) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const size_t base = ((size_t)mt * nblk + blk) * 4096;
        st.v[mt][0] = load16(xh + base); st.v[mt][1] = load16(xh + base + 2048);
        st.v[mt][2] = load16(xl + base); st.v[mt][3] = load16(xl + base + 2048);
    }
}

template <int MT>
__device__ __forceinline__ void gemm_b_store(const BStage<MT>& st, uint4* buf, int tid, bool live) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            uint4 v = st.v[mt][h];
            v.x = live ? v.x : 0u; v.y = live ? v.y : 0u; v.z = live ? v.z : 0u; v.w = live ? v.w : 0u;
            buf[(mt * 2 + (h >> 1)) * 512 + (h & 1) * 256 + tid] = v;
        }
}

// Transposes the weight tile into operand order through the wave's LDS tile (32 rows x 16 chunks of
// 16 bytes, chunk c of row r stored at chunk position c ^ (r & 15)), then multiplies it with the
// activation tile in `bt` ([mt][hi | lo][k-step][lane]).
template <int MT>
__device__ __forceinline__ void gemm_tile_mma(const uint4 (&ta)[8], f32x16 (&acc)[MT], uint4* at, const uint4* bt, int lane) {
    {
        const int r0 = lane >> 4, c = lane & 15;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int r = 4 * q + r0;
            at[r * 16 + (c ^ (r & 15))] = ta[q];
        }
    }
    uint4 a[8];
    {
        const int i = lane & 31, gh = lane >> 5;
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = at[i * 16 + ((2 * k + gh) ^ (i & 15))];
    }
    // The activation operands of k-step k + 1 are read from LDS while the products of step k run (a wave is alone on
    // its SIMD: nothing else hides the LDS latency), and consecutive products go to different accumulators.
    uint4 b0[MT][2], b1[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { b0[mt][0] = bt[(mt * 2 + 0) * 512 + lane]; b0[mt][1] = bt[(mt * 2 + 1) * 512 + lane]; }
#pragma unroll
    for (int k = 0; k < 8; k += 2) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { b1[mt][0] = bt[(mt * 2 + 0) * 512 + (k + 1) * 64 + lane]; b1[mt][1] = bt[(mt * 2 + 1) * 512 + (k + 1) * 64 + lane]; }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma_bf16(a[k], b0[mt][0], acc[mt]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma_bf16(a[k], b0[mt][1], acc[mt]);
        __builtin_amdgcn_sched_barrier(0);
        if (k + 2 < 8) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) { b0[mt][0] = bt[(mt * 2 + 0) * 512 + (k + 2) * 64 + lane]; b0[mt][1] = bt[(mt * 2 + 1) * 512 + (k + 2) * 64 + lane]; }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma_bf16(a[k + 1], b1[mt][0], acc[mt]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma_bf16(a[k + 1], b1[mt][1], acc[mt]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// SWIGLU (S = 1 only): W holds the gate rows [0, N/2) and the up rows [N/2, N).  Wave-tile t = 4 blockIdx.x + wave
// takes `rp` <= 16 gate rows (columns t rp .. t rp + rp - 1 of the result) into tile rows 0..rp-1 and the matching up
// rows into tile rows 16..16+rp-1: in the accumulator layout a gate product and its up product then sit in the same
// lane (registers 4b + r and 4(b + 2) + r), and the wave writes silu(gate) * up as hi/lo planes in operand order
// (act_hi, act_lo; N/2 columns) without any exchange.  The tile rows beyond rp repeat row rp - 1 (cache hits, results
// dropped): the launcher picks rp so that the tiles divide evenly among the waves of the device (14 rows for
// F = 14336 on 256 compute units: 1024 tiles), which a fixed 16 or 32 rows per wave would not.
template <int MT, bool SWIGLU>
__global__ __launch_bounds__(256) void k_chunk_gemm(const bf16_t* __restrict__ W, int N, int K,
                                                    const bf16_t* __restrict__ Xhi, const bf16_t* __restrict__ Xlo,
                                                    float* __restrict__ P, size_t s_stride, int n_stride, int S,
                                                    bf16_t* __restrict__ act_hi, bf16_t* __restrict__ act_lo, int rp) {
    extern __shared__ uint4 gemm_lds[];             // [4 waves][512] weight tiles, then [2][MT][2][512] activation tiles
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint4* at = gemm_lds + wave * 512;
    uint4* bt = gemm_lds + 2048;
    constexpr int BT = MT * 2 * 512;                // chunks in one activation buffer
    const int n0 = SWIGLU ? (blockIdx.x * 4 + wave) * rp : blockIdx.x * 128 + wave * 32;     // SWIGLU: first gate row
    const int nr = SWIGLU ? max(0, min(rp, (N >> 1) - n0)) : 32;                              // SWIGLU: gate rows of this wave
    const int sp = blockIdx.y;
    const int nblk = K >> 7;
    const int b0 = (int)((unsigned)(nblk * sp) / (unsigned)S), b1 = (int)((unsigned)(nblk * (sp + 1)) / (unsigned)S);   // (K / 128) * S < 2^31
    const int nb = b1 - b0;

    const bf16_t* wlane = W + (size_t)(SWIGLU ? 0 : n0 + (lane >> 4)) * K + (lane & 15) * 8;   // row l/16 (+4q), chunk l%16
    const size_t wstep = (size_t)4 * K;
    const bf16_t* wrow[8];
    if (SWIGLU) {
        const int g0 = min(n0, (N >> 1) - 1);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int slot = 4 * (q & 3) + (lane >> 4);
            wrow[q] = wlane + (size_t)((q < 4 ? 0 : N >> 1) + g0 + min(slot, max(nr, 1) - 1)) * K;
        }
    }
    const bf16_t* xh = Xhi + tid * 8;
    const bf16_t* xl = Xlo + tid * 8;

    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

    if (nb > 0) {
        // The workgroups walk their k-blocks in rotated order, each starting somewhere else: workgroups that all
        // read column block 0 of their own rows at the same time (rows are a multiple of 8 KiB apart) load few memory
        // channels at a time, and how badly depends on where the matrix lies (measured on the gate/up product, whose
        // workgroups all start together: 42 to 52 us for the same shape at different addresses).  Block i of the
        // walk is b0 + (i + rot) mod nb; past the end the last block is read again (a cache hit).
        const int rot = (int)((blockIdx.x / 8 + (blockIdx.x & 7) * 4 + blockIdx.y * 3) % (unsigned)nb);
        auto blk = [&](int i) { const int x = min(i, nb - 1) + rot; return b0 + (x >= nb ? x - nb : x); };
        // Waits are in issue order, so the activation loads of block t+2 are issued before the weight loads of
        // the newest block: waiting for the activations of block t+1 (to store them) then leaves the two newest
        // weight tiles in flight.
        constexpr int RING = GemmRing<MT>::N;
        uint4 ring[RING][8];
        BStage<MT> st[2];
        gemm_b_load<MT>(st[0], xh, xl, nblk, blk(0));
        gemm_b_load<MT>(st[1], xh, xl, nblk, blk(1));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < RING - 1; ++u) {
            if (SWIGLU) gemm_a_load(ring[u], wrow, blk(u));
            else gemm_a_load(ring[u], wlane, wstep, blk(u));
        }
        gemm_b_store<MT>(st[0], bt, tid, true);
        __syncthreads();
        // unrolled over an even number of blocks, so that ring slot (u % RING) and activation buffer (u & 1) are static
        constexpr int UNROLL = RING % 2 ? 2 * RING : RING;
        for (int t = 0; t < nb; t += UNROLL) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int tt = t + u;                       // this block of the walk
                if (UNROLL > RING && tt >= nb) break;       // long unroll only: uniform exit, nothing below is conditional
                gemm_b_load<MT>(st[u & 1], xh, xl, nblk, blk(tt + 2));
                __builtin_amdgcn_sched_barrier(0);
                if (SWIGLU) gemm_a_load(ring[(u + RING - 1) % RING], wrow, blk(tt + RING - 1));
                else gemm_a_load(ring[(u + RING - 1) % RING], wlane, wstep, blk(tt + RING - 1));
                __builtin_amdgcn_sched_barrier(0);
                gemm_tile_mma<MT>(ring[u % RING], acc, at, bt + (u & 1) * BT, lane);
                __builtin_amdgcn_sched_barrier(0);
                gemm_b_store<MT>(st[(u + 1) & 1], bt + ((u + 1) & 1) * BT, tid, tt + 1 < nb);
                __syncthreads();
            }
        }
    }

    // lane (j, g) holds D[8b + 4g + r][j] in register 4b + r: four consecutive weight rows of token row j
    if (SWIGLU) {
        const int F = N >> 1;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int slot = 8 * b + 4 * (lane >> 5) + r;
                    if (slot < nr) {
                        const float gt = acc[mt][4 * b + r], up = acc[mt][4 * (b + 2) + r];
                        bf16_t hi, lo;
                        split_bf16(gt / (1.f + expf(-gt)) * up, hi, lo);
                        const size_t o = tiled_off(mt * 32 + (lane & 31), n0 + slot, F);
                        act_hi[o] = hi; act_lo[o] = lo;
                    }
                }
        return;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float* prow = P + sp * s_stride + (size_t)(mt * 32 + (lane & 31)) * n_stride + n0 + 4 * (lane >> 5);
#pragma unroll
        for (int b = 0; b < 4; ++b)
            *(float4*)(prow + 8 * b) = make_float4(acc[mt][4 * b], acc[mt][4 * b + 1], acc[mt][4 * b + 2], acc[mt][4 * b + 3]);
    }
}

// ---------------------------------------------------------------------------------------------
// wide GEMM on the matrix cores for passes of more than 96 rows (prefill, large batched steps)
// ---------------------------------------------------------------------------------------------
// Workgroup = NW waves on a tile of 128 weight rows x (32 NW MW) token rows and one run of k-blocks.  Beyond 96
// rows a pass is bound by the matrix cores, not by the weight stream, so the tile is shaped for operand reuse:
//  * every wave multiplies ALL 128 weight rows of the tile with its own MW row tiles (32 token rows each):
//    per 16-column k-step 4 weight operands and 2 MW activation operands (hi, lo) feed 8 MW products;
//  * the weight block (128 rows x 128 columns) is loaded once per workgroup (4 rows x 256 contiguous bytes
//    per instruction), transposed into operand order through a double-buffered, XOR-swizzled LDS tile that
//    the waves share: one barrier per k-block;
//  * the activations are already in operand order in global memory (tiled planes: one contiguous KiB per
//    wave-wide load) and go straight to registers through a ring of four 2-step units, three units ahead of
//    the products; no wave reads another wave's rows, so they never pass through LDS.
// Workgroups that share a weight tile (row blocks of one pass) get linear ids that land on the same XCD,
// next to each other in dispatch order, so the second reads the weights from that XCD's L2.

template <int MW> struct BUnit { uint4 v[MW][2][2]; };      // [row tile][k-step of the unit][hi | lo]

template <int MW>
__device__ __forceinline__ void wide_b_load(BUnit<MW>& b, const bf16_t* (&xh)[MW], const bf16_t* (&xl)[MW],
                                            int blk, int unit) {
#pragma unroll
    for (int j = 0; j < MW; ++j)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const size_t o = ((size_t)blk * 8 + unit * 2 + st) * 512;
            b.v[j][st][0] = load16(xh[j] + o);
            b.v[j][st][1] = load16(xl[j] + o);
        }
}

// weight operands of k-step k: all four 32-row tiles of the block in `at`
__device__ __forceinline__ void wide_a_read(uint4 (&a)[4], const uint4* at, int k, int lane) {
    const int i = lane & 31, gh = lane >> 5;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) a[nt] = at[nt * 512 + i * 16 + ((2 * k + gh) ^ (i & 15))];
}

template <int MW>
__device__ __forceinline__ void wide_step(const uint4 (&a)[4], const BUnit<MW>& b, int st, f32x16 (&acc)[4][MW]) {
#pragma unroll
    for (int pl = 0; pl < 2; ++pl)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int j = 0; j < MW; ++j) acc[nt][j] = mfma_bf16(a[nt], b.v[j][st][pl], acc[nt][j]);
}

//
// SWIGLU: W holds the gate rows [0, N/2) and the up rows [N/2, N) of a feed-forward block.  The workgroup
// takes 64 gate rows and the 64 up rows of the same columns (weight-row tiles 0, 1 and 2, 3), and its
// epilogue writes silu(gate) * up as hi/lo planes in operand order (act_hi, act_lo; N/2 columns) instead of
// the fp32 products: S must be 1.
template <int NW, int MW, bool SWIGLU>
__global__ __launch_bounds__(NW * 64) void k_chunk_gemm_wide(const bf16_t* __restrict__ W, int N, int K,
                                                             const bf16_t* __restrict__ Xhi, const bf16_t* __restrict__ Xlo,
                                                             float* __restrict__ P, size_t s_stride, int n_stride, int S, int MT,
                                                             bf16_t* __restrict__ act_hi, bf16_t* __restrict__ act_lo) {
    extern __shared__ uint4 gemm_lds[];             // [2 buffers][4 weight-row tiles][512]
    constexpr int QN = 32 / NW;                     // weight loads per thread and block: wave w stages rows (128 / NW) w ...
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = N >> 7, MY = (MT + NW * MW - 1) / (NW * MW);
    int ntile, my, sp;
    {
        int q = blockIdx.x;
        if ((tiles & 7) == 0) {                     // XCDs take workgroups round robin by linear id
            const int xcd = q & 7;
            q >>= 3;
            my = q % MY; q /= MY;
            ntile = (q % (tiles >> 3)) * 8 + xcd; sp = q / (tiles >> 3);
        } else {
            my = q % MY; q /= MY;
            ntile = q % tiles; sp = q / tiles;
        }
    }
    const int nblk = K >> 7;
    const int b0 = (int)((unsigned)(nblk * sp) / (unsigned)S), b1 = (int)((unsigned)(nblk * (sp + 1)) / (unsigned)S);   // (K / 128) * S < 2^31
    const int nb = b1 - b0, last = b1 - 1;
    const int n0 = ntile * 128;

    // weights: load q of a thread covers row (128 / NW) wave + 4 q + lane / 16 of the tile, 16-byte chunk lane % 16
    const bf16_t* wq[QN];
    int wslot[QN];
#pragma unroll
    for (int q = 0; q < QN; ++q) {
        const int rg = wave * (128 / NW) + 4 * q + (lane >> 4), r = rg & 31, c = lane & 15;
        const int row = SWIGLU ? (rg < 64 ? ntile * 64 + rg : (N >> 1) + ntile * 64 + rg - 64) : n0 + rg;
        wq[q] = W + (size_t)row * K + c * 8;
        wslot[q] = (rg >> 5) * 512 + r * 16 + (c ^ (r & 15));
    }
    // activations: row tiles (my MW + j) NW + wave of the pass; tiles past the end repeat the last one and are not stored
    int mtile[MW];
    const bf16_t* xh[MW];
    const bf16_t* xl[MW];
#pragma unroll
    for (int j = 0; j < MW; ++j) {
        mtile[j] = (my * MW + j) * NW + wave;
        const size_t o = (size_t)min(mtile[j], MT - 1) * nblk * 4096 + lane * 8;
        xh[j] = Xhi + o; xl[j] = Xlo + o;
    }

    f32x16 acc[4][MW];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int j = 0; j < MW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][j][r] = 0.f;

    if (nb > 0) {
        uint4 wreg[QN];
        BUnit<MW> ring[4];
        auto w_load = [&](int blk) {
#pragma unroll
            for (int q = 0; q < QN; ++q) wreg[q] = load16_stream(wq[q] + (size_t)blk * 128);
        };
        auto w_store = [&](uint4* at) {
#pragma unroll
            for (int q = 0; q < QN; ++q) at[wslot[q]] = wreg[q];
        };
        // issue order = completion order: weights of the first block, three activation units, weights of the second block
        w_load(b0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 3; ++u) wide_b_load<MW>(ring[u], xh, xl, b0, u);
        __builtin_amdgcn_sched_barrier(0);
        w_store(gemm_lds);
        w_load(min(b0 + 1, last));
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        for (int t = 0; t < nb; t += 2) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tt = b0 + t + h;                  // this block, in LDS buffer h
                if (tt > last) break;                       // uniform
                const uint4* at = gemm_lds + h * 2048;
                uint4 a0[4], a1[4];
                wide_a_read(a0, at, 0, lane);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // unit u + 3 of the stream: the last unit of this block, then the first three of the next
                    wide_b_load<MW>(ring[(u + 3) & 3], xh, xl, u == 0 ? tt : min(tt + 1, last), (u + 3) & 3);
                    __builtin_amdgcn_sched_barrier(0);
                    if (u == 1) {
                        // the next block's weights (requested one block ago) move to the other LDS buffer, whose
                        // readers passed the barrier that ended the previous block; then the block after is requested
                        w_store(gemm_lds + (h ^ 1) * 2048);
                        w_load(min(tt + 2, last));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    wide_a_read(a1, at, 2 * u + 1, lane);
                    __builtin_amdgcn_sched_barrier(0);
                    wide_step<MW>(a0, ring[u], 0, acc);
                    __builtin_amdgcn_sched_barrier(0);
                    if (u < 3) wide_a_read(a0, at, 2 * u + 2, lane);
                    __builtin_amdgcn_sched_barrier(0);
                    wide_step<MW>(a1, ring[u], 1, acc);
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();
            }
        }
    }

    // lane (j, g) holds D[8b + 4g + r][j] in register 4b + r: four consecutive weight rows of token row j
    if (SWIGLU) {
        const int F = N >> 1, f0 = ntile * 64 + 4 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < MW; ++j) {
            if (mtile[j] >= MT) continue;
            const int m = mtile[j] * 32 + (lane & 31);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    bf16_t hi[4], lo[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float gt = acc[nt][j][4 * b + r], up = acc[nt + 2][j][4 * b + r];
                        split_bf16(gt / (1.f + expf(-gt)) * up, hi[r], lo[r]);
                    }
                    const size_t o = tiled_off(m, f0 + nt * 32 + 8 * b, F);     // four columns inside one 8-element group
                    *reinterpret_cast<uint2*>(act_hi + o) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                    *reinterpret_cast<uint2*>(act_lo + o) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
                }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < MW; ++j) {
        if (mtile[j] >= MT) continue;
        float* prow = P + sp * s_stride + (size_t)(mtile[j] * 32 + (lane & 31)) * n_stride + n0 + 4 * (lane >> 5);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                *(float4*)(prow + nt * 32 + 8 * b) = make_float4(acc[nt][j][4 * b], acc[nt][j][4 * b + 1], acc[nt][j][4 * b + 2], acc[nt][j][4 * b + 3]);
    }
}

// ---------------------------------------------------------------------------------------------
// GEMM for passes of 33-64 rows: the four waves of a workgroup split the k-steps
// ---------------------------------------------------------------------------------------------
// With two row tiles k_chunk_gemm is bound by LDS: a wave that owns 32 weight rows uses every activation
// operand it reads for one product only.  Here every wave multiplies the whole tile of the workgroup, 128 weight
// rows x all MT row tiles, but only for two of the eight 16-column steps of each k-block (wave w: steps 2w, 2w+1):
// per step 4 weight operands (from the shared LDS tile, staged as in k_chunk_gemm_wide) and 2 MT activation
// operands (straight from the operand-order planes, two blocks ahead) feed 8 MT products, and no operand
// is read by two waves.  The four partial tiles are added through LDS at the end, in wave order.

template <int MT, bool SWIGLU>
__global__ __launch_bounds__(256) void k_chunk_gemm_ks(const bf16_t* __restrict__ W, int N, int K,
                                                       const bf16_t* __restrict__ Xhi, const bf16_t* __restrict__ Xlo,
                                                       float* __restrict__ P, size_t s_stride, int n_stride, int S,
                                                       bf16_t* __restrict__ act_hi, bf16_t* __restrict__ act_lo) {
    extern __shared__ uint4 gemm_lds[];             // [2 buffers][4 weight-row tiles][512]; reused by the final sum
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ntile = blockIdx.x, sp = blockIdx.y;
    const int nblk = K >> 7;
    const int b0 = (int)((unsigned)(nblk * sp) / (unsigned)S), b1 = (int)((unsigned)(nblk * (sp + 1)) / (unsigned)S);   // (K / 128) * S < 2^31
    const int nb = b1 - b0;
    const int n0 = ntile * 128;

    // weights: load q of a thread covers row 32 wave + 4 q + lane / 16 of the tile, 16-byte chunk lane % 16
    const int wrow = SWIGLU ? (wave < 2 ? ntile * 64 + wave * 32 : (N >> 1) + ntile * 64 + (wave - 2) * 32) : n0 + wave * 32;
    const bf16_t* wlane = W + (size_t)(wrow + (lane >> 4)) * K + (lane & 15) * 8;
    const size_t wstep = (size_t)4 * K;
    const int wr0 = lane >> 4, wc = lane & 15;
    const bf16_t* xh[MT];
    const bf16_t* xl[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        const size_t o = (size_t)j * nblk * 4096 + lane * 8;
        xh[j] = Xhi + o; xl[j] = Xlo + o;
    }

    f32x16 acc[4][MT];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][j][r] = 0.f;

    if (nb > 0) {
        // A block is short (32 products per wave with two row tiles), so the weights of block b0 + i travel in register
        // set i % 2, requested two blocks ahead of their use, and the activations (from L2) in a ring of three blocks.
        // (Three row tiles do not fit the register file this way; they take k_chunk_gemm_wide with an idle wave.)
        static_assert(MT == 2, "register budget");
        // rotated walk over the k-blocks, as in k_chunk_gemm: block i of the walk is b0 + (i + rot) mod nb
        const int rot = (int)((blockIdx.x / 8 + (blockIdx.x & 7) * 4 + blockIdx.y * 3) % (unsigned)nb);
        auto blk = [&](int i) { const int x = min(i, nb - 1) + rot; return b0 + (x >= nb ? x - nb : x); };
        constexpr int NSET = 2, RING = 3, UNROLL = 6;   // LDS buffer u % 2 and ring slot u % RING are static
        uint4 wreg[NSET][8];
        BUnit<MT> ring[RING];
        auto w_load = [&](uint4 (&set)[8], int blk) { gemm_a_load(set, wlane, wstep, blk); };
        auto w_store = [&](const uint4 (&set)[8], uint4* at) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int r = 4 * q + wr0;
                at[wave * 512 + r * 16 + (wc ^ (r & 15))] = set[q];
            }
        };
        // issue order = completion order: weights of the first block, activations of the first two, weights of the second
        w_load(wreg[0], blk(0));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < RING - 1; ++i) wide_b_load<MT>(ring[i], xh, xl, blk(i), wave);
        __builtin_amdgcn_sched_barrier(0);
        w_store(wreg[0], gemm_lds);
        w_load(wreg[NSET - 1], blk(1));
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        for (int t = 0; t < nb; t += UNROLL) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int tt = t + u;                       // this block of the walk: LDS buffer u % 2, ring slot u % RING
                if (tt >= nb) break;                        // uniform
                const uint4* at = gemm_lds + (u & 1) * 2048;
                uint4* other = gemm_lds + ((u & 1) ^ 1) * 2048;   // its readers passed the barrier that ended the previous block
                wide_b_load<MT>(ring[(u + RING - 1) % RING], xh, xl, blk(tt + RING - 1), wave);
                __builtin_amdgcn_sched_barrier(0);
                w_load(wreg[u & 1], blk(tt + 2));           // this set's previous block was stored one block ago
                __builtin_amdgcn_sched_barrier(0);
                uint4 a0[4], a1[4];
                wide_a_read(a0, at, 2 * wave, lane);
                wide_a_read(a1, at, 2 * wave + 1, lane);
                __builtin_amdgcn_sched_barrier(0);
                wide_step<MT>(a0, ring[u % RING], 0, acc);
                __builtin_amdgcn_sched_barrier(0);
                wide_step<MT>(a1, ring[u % RING], 1, acc);
                __builtin_amdgcn_sched_barrier(0);
                w_store(wreg[(u + 1) & 1], other);          // the next block's weights, requested two blocks ago
                __syncthreads();
            }
        }
    }

    // sum of the four waves' partial tiles, one row tile at a time: [wave][weight-row tile][register quad][lane] float4
    float4* ex = reinterpret_cast<float4*>(gemm_lds);
#pragma unroll
    for (int j = 0; j < MT; ++j) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                ex[((wave * 4 + nt) * 4 + b) * 64 + lane] = make_float4(acc[nt][j][4 * b], acc[nt][j][4 * b + 1], acc[nt][j][4 * b + 2], acc[nt][j][4 * b + 3]);
        __syncthreads();
        // lane (j, g) holds D[8b + 4g + r][j] in register 4b + r: four consecutive weight rows of token row j
        const int m = j * 32 + (lane & 31);
        if (SWIGLU) {
            if (wave < 2) {                                 // wave w: gate tile w and up tile w + 2
                const int F = N >> 1, f0 = ntile * 64 + wave * 32 + 4 * (lane >> 5);
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    float4 gt = ex[((0 * 4 + wave) * 4 + b) * 64 + lane], up = ex[((0 * 4 + wave + 2) * 4 + b) * 64 + lane];
#pragma unroll
                    for (int w = 1; w < 4; ++w) {
                        const float4 g2 = ex[((w * 4 + wave) * 4 + b) * 64 + lane], u2 = ex[((w * 4 + wave + 2) * 4 + b) * 64 + lane];
                        gt.x += g2.x; gt.y += g2.y; gt.z += g2.z; gt.w += g2.w;
                        up.x += u2.x; up.y += u2.y; up.z += u2.z; up.w += u2.w;
                    }
                    const float gv[4] = {gt.x, gt.y, gt.z, gt.w}, uv[4] = {up.x, up.y, up.z, up.w};
                    bf16_t hi[4], lo[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) split_bf16(gv[r] / (1.f + expf(-gv[r])) * uv[r], hi[r], lo[r]);
                    const size_t o = tiled_off(m, f0 + 8 * b, F);       // four columns inside one 8-element group
                    *reinterpret_cast<uint2*>(act_hi + o) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                    *reinterpret_cast<uint2*>(act_lo + o) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
                }
            }
        } else {                                            // wave w: weight-row tile w
            float* prow = P + sp * s_stride + (size_t)m * n_stride + n0 + wave * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float4 v = ex[((0 * 4 + wave) * 4 + b) * 64 + lane];
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const float4 v2 = ex[((w * 4 + wave) * 4 + b) * 64 + lane];
                    v.x += v2.x; v.y += v2.y; v.z += v2.z; v.w += v2.w;
                }
                *(float4*)(prow + 8 * b) = v;
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// causal chunk attention on the matrix cores (head_dim 128, paired bf16 cache)
// ---------------------------------------------------------------------------------------------
// One wave = one (task, kv head, key split); a task is a tile of 32 query columns of one group, the columns
// of a group being (q head within the kv group, row) pairs, so a single-row group of a 4:1 model fills
// 4 columns and a 24-row group three tiles.  Per 32-key tile the wave loads K and V^T (both planes) at once,
// forms S^T = K Q^T (keys along D rows), does the online softmax per query column, and accumulates
// O^T += V^T P^T.  Key rows are permuted so that the D registers of a lane hold 16 consecutive keys, which
// makes P directly usable as the next B operand.

struct ChunkAttnArgs {
    const bf16_t* q_hi; const bf16_t* q_lo;     // [Hkv][q_cols][128], scaled by 1/sqrt(dh)
    const bf16_t* kv_layer;
    const ChunkTable* tab;
    float* part_o;      // [unit][128][32]
    float* part_ml;     // [unit][2][32]
    int32_t nsplit, q_cols;
};

// K tile (32 keys x 128 channels, one plane) as loaded: instruction q covers rows 4q .. 4q+3, lane l holds
// row 4q + l/16, 16-byte chunk l%16 (1 KiB contiguous per instruction).
__device__ __forceinline__ void attn_k_load(uint4 (&kh)[8], uint4 (&kl)[8], const bf16_t* Kp, size_t lo, int key0, int lane) {
    const bf16_t* p = Kp + (size_t)(key0 + (lane >> 4)) * 128 + (lane & 15) * 8;
#pragma unroll
    for (int q = 0; q < 8; ++q) { kh[q] = load16(p + q * 512); kl[q] = load16(p + lo + q * 512); }
}

// V^T tile (both planes) in operand order: instruction (dt, t) is one contiguous KiB in lane order.
__device__ __forceinline__ void attn_v_load(uint4 (&vh)[8], uint4 (&vl)[8], const bf16_t* Vt, size_t lo, int tile, int lane) {
    const bf16_t* p = Vt + ((size_t)tile * 8 * 64 + lane) * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) { vh[k] = load16(p + k * 512); vl[k] = load16(p + lo + k * 512); }
}

// chunk position of 16-byte chunk c of row r in the wave's LDS tile (conflict-free for the row-wise writes and
// for the reads of the permuted key rows)
__device__ __forceinline__ int attn_k_slot(int r, int c) { return r * 16 + (c ^ ((r & 7) | ((r >> 1) & 8))); }

struct AttnState {
    f32x16 o[4];
    float mrun, lrun;
};

// One 32-key tile: K goes through the wave's LDS tile (attn_stage_k) into A-operand order (key rows permuted so
// that the D registers of a lane hold 16 consecutive keys), then S^T = K Q^T, online softmax, O^T += V^T P^T.
__device__ __forceinline__ void attn_stage_k(const uint4 (&kh)[8], const uint4 (&kl)[8], uint4* kt, int lane) {
    const int r0 = lane >> 4, c = lane & 15;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        kt[attn_k_slot(4 * q + r0, c)] = kh[q];
        kt[512 + attn_k_slot(4 * q + r0, c)] = kl[q];
    }
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> two bf16 (round to nearest even) in one 32-bit word, first value in the low half (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float x, float y) {
    const f32x2 v = {x, y};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// hi = bf16(p), lo = bf16(p - hi) for a pair of values
__device__ __forceinline__ void split_pair(float x, float y, uint32_t& hi, uint32_t& lo) {
    hi = pack_bf16x2(x, y);
    lo = pack_bf16x2(x - __uint_as_float(hi << 16), y - __uint_as_float(hi & 0xffff0000u));
}

// The per-tile arithmetic outside the matrix cores is what bounds this kernel (a wave is alone on its SIMD and every
// vector instruction takes four cycles), so it is kept short: packed conversions, exp through the hardware exp2,
// and the two steps that most tiles do not need (causal mask away from the diagonal, rescaling of the output when
// no column's maximum moved) are skipped on a wave-uniform test.
__device__ __forceinline__ void attn_tile(AttnState& st, const uint4 (&vh)[8], const uint4 (&vl)[8], const uint4 (&qh)[8],
                                          const uint4 (&ql)[8], const uint4* kt, int key0, int qpos, int lane) {
    const int i = lane & 31, gh = lane >> 5;
    const int krow = (i >> 3) * 4 + (i & 3) + 16 * ((i >> 2) & 1);   // key (within the tile) held in A row i
    // hi.hi + lo.hi + hi.lo accumulate into one register set (back-to-back accumulation), K operands read from LDS
    // two steps ahead
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    uint4 kq[3][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) { kq[j][0] = kt[attn_k_slot(krow, 2 * j + gh)]; kq[j][1] = kt[512 + attn_k_slot(krow, 2 * j + gh)]; }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if (t + 2 < 8) {
            kq[(t + 2) % 3][0] = kt[attn_k_slot(krow, 2 * (t + 2) + gh)];
            kq[(t + 2) % 3][1] = kt[512 + attn_k_slot(krow, 2 * (t + 2) + gh)];
        }
        __builtin_amdgcn_sched_barrier(0);
        s = mfma_bf16(kq[t % 3][0], qh[t], s);
        s = mfma_bf16(kq[t % 3][1], qh[t], s);
        s = mfma_bf16(kq[t % 3][0], ql[t], s);
        __builtin_amdgcn_sched_barrier(0);
    }
    // register r of lane (j, g) is key key0 + 16 g + r for query column j
    if (__builtin_amdgcn_ballot_w64(key0 + 31 > qpos) != 0) {        // the tile reaches past some column's position
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (key0 + 16 * gh + r > qpos) s[r] = -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mnew = fmaxf(st.mrun, mx);
    const float msafe = mnew == -INFINITY ? 0.f : mnew;
    const float corr = __expf(st.mrun - msafe);
    float psum = 0.f;
    uint32_t ph[8], pl[8];
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
        const float p0 = __expf(s[r] - msafe), p1 = __expf(s[r + 1] - msafe);
        psum += p0 + p1;
        split_pair(p0, p1, ph[r >> 1], pl[r >> 1]);
    }
    st.lrun = st.lrun * corr + psum;
    if (__builtin_amdgcn_ballot_w64(mnew != st.mrun) != 0) {          // some column's running maximum moved
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[dt][r] *= corr;
    }
    st.mrun = mnew;
    // consecutive products go to different accumulators
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const uint4 pht = make_uint4(ph[4 * t], ph[4 * t + 1], ph[4 * t + 2], ph[4 * t + 3]);
        const uint4 plt = make_uint4(pl[4 * t], pl[4 * t + 1], pl[4 * t + 2], pl[4 * t + 3]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) st.o[dt] = mfma_bf16(vh[dt * 2 + t], pht, st.o[dt]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) st.o[dt] = mfma_bf16(vl[dt * 2 + t], pht, st.o[dt]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) st.o[dt] = mfma_bf16(vh[dt * 2 + t], plt, st.o[dt]);
    }
}

__global__ __launch_bounds__(256) void k_chunk_attn(ChunkAttnArgs a, Geom g) {
    constexpr int DH = 128;
    extern __shared__ uint4 attn_lds[];                    // [4 waves][hi | lo][512 chunks] K tiles
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, gh = lane >> 5;
    uint4* kt = attn_lds + wave * 1024;
    const int G = g.Hq / g.Hkv;
    const int kvh = blockIdx.x % g.Hkv, split = blockIdx.y * (int)(blockDim.x >> 6) + wave;
    const ChunkTask T = a.tab->task[blockIdx.x / g.Hkv];
    // Columns 32 tile .. 32 tile + 31 of the group are rows first .. first + 31 of one query head, or wrap into the
    // next head (then the group's last row is among them): no column of the tile sees keys past its latest row.
    const int first = (32 * T.tile) % T.n;
    const int Lk = T.pos0 + min(first + 32, T.n);          // keys 0 .. Lk-1 matter to this tile
    const int ntile = (Lk + 31) >> 5;
    const int tps = (ntile + a.nsplit - 1) / a.nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    const size_t seq_off = (size_t)T.seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
    const bf16_t* Kp = a.kv_layer + seq_off;
    const bf16_t* Vt = a.kv_layer + g.kv_vt_offset + seq_off;
    const size_t lo = g.kv_lo_offset;

    // this lane's query column: (q head, row r) of the group; columns past the group are computed and dropped
    const int col = 32 * T.tile + i;
    const int qpos = T.pos0 + col % T.n;

    AttnState st;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
    st.mrun = -INFINITY; st.lrun = 0.f;

    if (t0 < t1) {
        // B operand of S^T = K Q^T: lane (j, g) holds q[j][16 t + 8 g + e]
        uint4 qh[8], ql[8];
        {
            const size_t qo = ((size_t)kvh * a.q_cols + (size_t)G * T.row0 + col) * DH + gh * 8;
#pragma unroll
            for (int t = 0; t < 8; ++t) { qh[t] = load16(a.q_hi + qo + t * 16); ql[t] = load16(a.q_lo + qo + t * 16); }
        }
        // Once K of a tile is staged in LDS its registers take K of the next tile (clamped to the last one), and the V
        // registers take the next tile's V as soon as the P V product has used them, so the next tile's loads are in
        // flight while a tile is multiplied.  No conditional code around loads or their uses (the compiler would
        // sink the loads next to the uses).
        uint4 kh[8], kl[8], vh[8], vl[8];
        __builtin_amdgcn_sched_barrier(0);          // issue order q, K, V: the waits in the loop count on it
        attn_k_load(kh, kl, Kp, lo, t0 * 32, lane);
        __builtin_amdgcn_sched_barrier(0);
        attn_v_load(vh, vl, Vt, lo, t0, lane);
        __builtin_amdgcn_sched_barrier(0);
        for (int tile = t0; tile < t1; ++tile) {
            const int n1 = min(tile + 1, t1 - 1);
            attn_stage_k(kh, kl, kt, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_k_load(kh, kl, Kp, lo, n1 * 32, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_tile(st, vh, vl, qh, ql, kt, tile * 32, qpos, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_v_load(vh, vl, Vt, lo, n1, lane);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    st.lrun += __shfl_xor(st.lrun, 32, 64);

    const size_t unit = (size_t)blockIdx.x * a.nsplit + split;
    float* po = a.part_o + unit * DH * 32;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r2 = 0; r2 < 16; ++r2) po[(size_t)(dt * 32 + 8 * (r2 >> 2) + 4 * gh + (r2 & 3)) * 32 + i] = st.o[dt][r2];
    if (gh == 0) {
        float* pm = a.part_ml + unit * 64;
        pm[i] = st.mrun; pm[32 + i] = st.lrun;
    }
}

// ---------------------------------------------------------------------------------------------
// single-row decoding attention on the matrix cores, one kernel
// ---------------------------------------------------------------------------------------------
// grid (Hkv, nsplit / waves per workgroup); wave = (kv head, key split), the q heads of the kv group are the first G query columns
// of the tile (the other columns are zero and dropped).  Keys and values of the wave's first tile are requested
// first, then the step's fp32 query, which is split into bf16 pairs while they arrive.  Each wave leaves the G
// useful columns of its partial result ([G][128] + running maximum and sum); k_decode_attn_merge, a kernel of its
// own, merges the splits that had keys.  (Merging in the same kernel by the workgroup that finishes last needs two
// device-wide fences and a ticket before the partial results can be read, a longer chain than a kernel boundary.)
struct DecodeAttnArgs {
    const float* q;             // [Hq][128] rotated, unscaled
    const StepDesc* step;
    const bf16_t* kv_layer;
    float* part_o;              // [Hkv][nsplit][G][128]
    float* part_ml;             // [Hkv][nsplit][2][G]
    float* out;                 // [Hq][128]
    int32_t nsplit;
    unsigned long long* stamps; // stamp mode of the one-stream step: six words for this kernel, six for the merge
    unsigned long long* done_wg; // ... and STAMP_DONE_SLOTS finishing-time words each
};

__global__ __launch_bounds__(256) void k_decode_attn_mfma(DecodeAttnArgs a, Geom g) {
    constexpr int DH = 128;
    extern __shared__ uint4 attn_lds[];                    // [4 waves][hi | lo][512 chunks] K tiles
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    PipeSync stamp{};
    stamp.stamps = a.stamps; stamp.done_wg = a.done_wg;
    const unsigned long long t_start = clock_if(stamp.done_wg != nullptr);
    const int i = lane & 31, gh = lane >> 5;
    uint4* kt = attn_lds + wave * 1024;
    const int G = g.Hq / g.Hkv;
    const int kvh = blockIdx.x, split = blockIdx.y * (int)(blockDim.x >> 6) + wave, nsplit = a.nsplit;
    const int seq = a.step->seq, pos = a.step->pos;
    const int ntile = (pos + 32) >> 5;                     // keys 0 .. pos
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    const size_t seq_off = (size_t)seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
    const bf16_t* Kp = a.kv_layer + seq_off;
    const bf16_t* Vt = a.kv_layer + g.kv_vt_offset + seq_off;
    const size_t lo = g.kv_lo_offset;

    if (t0 < t1) {
        AttnState st;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
        st.mrun = -INFINITY; st.lrun = 0.f;
        uint4 kh[8], kl[8], vh[8], vl[8];
        __builtin_amdgcn_sched_barrier(0);          // issue order K, V, q: the waits in the loop count on it
        attn_k_load(kh, kl, Kp, lo, t0 * 32, lane);
        __builtin_amdgcn_sched_barrier(0);
        attn_v_load(vh, vl, Vt, lo, t0, lane);
        __builtin_amdgcn_sched_barrier(0);
        // B operand of S^T = K Q^T: lane (j, g) holds q[j][16 t + 8 g + e]; column j is q head j of the kv group
        uint4 qh[8], ql[8];
        {
            const float* qp = a.q + (size_t)(kvh * G + min(i, G - 1)) * DH + gh * 8;
            const float sc = i < G ? g.scale : 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float4 v0 = *reinterpret_cast<const float4*>(qp + t * 16), v1 = *reinterpret_cast<const float4*>(qp + t * 16 + 4);
                split_pair(v0.x * sc, v0.y * sc, qh[t].x, ql[t].x); split_pair(v0.z * sc, v0.w * sc, qh[t].y, ql[t].y);
                split_pair(v1.x * sc, v1.y * sc, qh[t].z, ql[t].z); split_pair(v1.z * sc, v1.w * sc, qh[t].w, ql[t].w);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        for (int tile = t0; tile < t1; ++tile) {
            const int n1 = min(tile + 1, t1 - 1);
            attn_stage_k(kh, kl, kt, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_k_load(kh, kl, Kp, lo, n1 * 32, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_tile(st, vh, vl, qh, ql, kt, tile * 32, pos, lane);
            __builtin_amdgcn_sched_barrier(0);
            attn_v_load(vh, vl, Vt, lo, n1, lane);
            __builtin_amdgcn_sched_barrier(0);
        }
        st.lrun += __shfl_xor(st.lrun, 32, 64);
        if (i < G) {
            // register r2 of accumulator dt is channel 32 dt + 8 (r2 / 4) + 4 gh + r2 % 4 of column i
            const size_t unit = (size_t)kvh * nsplit + split;
            float* po = a.part_o + (unit * G + i) * DH + 4 * gh;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<float4*>(po + dt * 32 + 8 * q4) =
                        make_float4(st.o[dt][4 * q4], st.o[dt][4 * q4 + 1], st.o[dt][4 * q4 + 2], st.o[dt][4 * q4 + 3]);
            if (gh == 0) {
                float* pm = a.part_ml + unit * 2 * G;
                pm[i] = st.mrun; pm[G + i] = st.lrun;
            }
        }
    }
    step_stamp_done(stamp, t_start, 0);
}

// Merge of the key splits: grid (Hkv, G * 128 / 64), a workgroup writes 64 of the kv group's G x 128 outputs.  Thread =
// (output, quarter of the splits): the splits are few long chains of loads otherwise (96 splits at a long context), the
// four partial sums of an output meet in LDS and are added in a fixed order.
__global__ __launch_bounds__(256) void k_decode_attn_merge(DecodeAttnArgs a, Geom g) {
    constexpr int DH = 128;
    __shared__ float f[8 * CHUNK_ATTN_MAX_SPLIT];          // [G][nused] weights exp(m_s - M) / L
    __shared__ float red[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    PipeSync stamp{};
    stamp.stamps = a.stamps ? a.stamps + 6 : nullptr; stamp.done_wg = a.done_wg ? a.done_wg + STAMP_DONE_SLOTS : nullptr;
    const unsigned long long t_start = clock_if(stamp.done_wg != nullptr);
    const int G = g.Hq / g.Hkv;
    const int kvh = blockIdx.x, nsplit = a.nsplit;
    const int ntile = (a.step->pos + 32) >> 5;
    const int tps = (ntile + nsplit - 1) / nsplit;
    const int nused = (ntile + tps - 1) / tps;             // splits that had keys
    const float* ml = a.part_ml + (size_t)kvh * nsplit * 2 * G;
    const int per = (G * DH + (int)gridDim.y - 1) / (int)gridDim.y;
    const int o0 = blockIdx.y * per, o1 = min(o0 + per, G * DH);
    for (int gq = (o0 >> 7) + wave; gq <= ((o1 - 1) >> 7); gq += 4) {      // the q heads this workgroup writes; lanes over splits
        float M = -INFINITY;
        for (int sp = lane; sp < nused; sp += 64) M = fmaxf(M, ml[sp * 2 * G + gq]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
        float L = 0.f;
        for (int sp = lane; sp < nused; sp += 64) {
            const float m = ml[sp * 2 * G + gq];
            const float w = m > -INFINITY ? expf(m - M) : 0.f;
            L += ml[sp * 2 * G + G + gq] * w;
            f[gq * nused + sp] = w;
        }
        L = wave_sum(L);
        const float inv = L > 0.f ? 1.f / L : 0.f;
        for (int sp = lane; sp < nused; sp += 64) f[gq * nused + sp] *= inv;
    }
    __syncthreads();
    for (int base = o0; base < o1; base += 64) {
        const int idx = base + lane;
        float acc = 0.f;
        if (idx < o1) {
            const int gq = idx >> 7, ch = idx & (DH - 1);
            const float* po = a.part_o + ((size_t)kvh * nsplit * G + gq) * DH + ch;
            const float* fw = f + gq * nused;
#pragma unroll 8
            for (int sp = wave; sp < nused; sp += 4) acc = fmaf(po[(size_t)sp * G * DH], fw[sp], acc);
        }
        red[tid] = acc;
        __syncthreads();
        if (wave == 0 && idx < o1)
            a.out[(size_t)kvh * G * DH + idx] = (red[lane] + red[64 + lane]) + (red[128 + lane] + red[192 + lane]);
        __syncthreads();
    }
    step_stamp_done(stamp, t_start, 0);
}

// ---------------------------------------------------------------------------------------------
// the same attention for large groups (prefill, long interrupts): keys and values shared by four tasks
// ---------------------------------------------------------------------------------------------
// Workgroup = (block of up to four consecutive tasks of one group, kv head, key split); wave w works on task w of
// the block (128 query columns per workgroup).  The K and V^T tiles of 32 keys (both planes, 32 KiB) are loaded once
// per workgroup, 8 x 16 bytes per thread, into a double-buffered LDS tile while the previous tile is multiplied:
// K in the swizzled row layout of attn_stage_k, V^T verbatim (it is stored in operand order), and all four waves
// read their operands from there.  Against one wave per task this divides the traffic from L2 by four, which is
// what bounds a 512-row pass over a long context.  Partial results go to the same units as k_chunk_attn writes, so
// k_chunk_attn_combine serves both.

struct WideTileRegs { uint4 k[4], v[4]; };   // this thread's share of a tile: K hi, hi, lo, lo; V^T hi, hi, lo, lo

__device__ __forceinline__ void attn_wide_load(WideTileRegs& r, const bf16_t* Kp, const bf16_t* Vt, size_t lo, int tile, int tid) {
    // K: chunk c = tid + 256 h is row c / 16, 16-byte piece c % 16 of the tile; V^T: chunk c of the tile's contiguous 8 KiB
    const bf16_t* kp = Kp + (size_t)tile * 32 * 128 + (size_t)tid * 8;
    const bf16_t* vp = Vt + ((size_t)tile * 512 + tid) * 8;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        r.k[h] = load16(kp + h * 2048); r.k[2 + h] = load16(kp + lo + h * 2048);
        r.v[h] = load16(vp + h * 2048); r.v[2 + h] = load16(vp + lo + h * 2048);
    }
}

// buffer layout (16-byte chunks): K hi [0, 512), K lo [512, 1024), V^T hi [1024, 1536), V^T lo [1536, 2048)
__device__ __forceinline__ void attn_wide_store(const WideTileRegs& r, uint4* buf, int tid) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = (tid >> 4) + 16 * h, c = tid & 15;
        buf[attn_k_slot(row, c)] = r.k[h];
        buf[512 + attn_k_slot(row, c)] = r.k[2 + h];
        buf[1024 + tid + 256 * h] = r.v[h];
        buf[1536 + tid + 256 * h] = r.v[2 + h];
    }
}

__global__ __launch_bounds__(256) void k_chunk_attn_wide(ChunkAttnArgs a, Geom g) {
    constexpr int DH = 128;
    extern __shared__ uint4 attn_lds[];                    // [2 buffers][2048 chunks]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 31, gh = lane >> 5;
    const int G = g.Hq / g.Hkv;
    const int kvh = blockIdx.x % g.Hkv, split = blockIdx.y;
    const ChunkTaskBlock B = a.tab->block[blockIdx.x / g.Hkv];
    const bool live = wave < B.n;
    const int task = B.task0 + min(wave, B.n - 1);
    const ChunkTask T0 = a.tab->task[B.task0];
    const ChunkTask T = a.tab->task[task];
    // keys that matter to the block's columns (its tasks are consecutive tiles of one group), split evenly
    const int Lk = T0.pos0 + min((32 * T0.tile) % T0.n + 32 * B.n, T0.n);
    const int ntile = (Lk + 31) >> 5;
    const int tps = (ntile + a.nsplit - 1) / a.nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);
    // and to this wave's own columns: later tiles are loaded for the other waves but not multiplied here
    const int Lw = T.pos0 + min((32 * T.tile) % T.n + 32, T.n);

    const size_t seq_off = (size_t)T.seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
    const bf16_t* Kp = a.kv_layer + seq_off;
    const bf16_t* Vt = a.kv_layer + g.kv_vt_offset + seq_off;
    const size_t lo = g.kv_lo_offset;
    const int col = 32 * T.tile + i;
    const int qpos = T.pos0 + col % T.n;

    AttnState st;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[dt][r] = 0.f;
    st.mrun = -INFINITY; st.lrun = 0.f;

    if (t0 < t1) {
        uint4 qh[8], ql[8];
        {
            const size_t qo = ((size_t)kvh * a.q_cols + (size_t)G * T.row0 + col) * DH + gh * 8;
#pragma unroll
            for (int t = 0; t < 8; ++t) { qh[t] = load16(a.q_hi + qo + t * 16); ql[t] = load16(a.q_lo + qo + t * 16); }
        }
        WideTileRegs regs;
        __builtin_amdgcn_sched_barrier(0);
        attn_wide_load(regs, Kp, Vt, lo, t0, tid);
        attn_wide_store(regs, attn_lds, tid);
        __syncthreads();
        for (int tile = t0; tile < t1; ++tile) {
            uint4* buf = attn_lds + ((tile - t0) & 1) * 2048;
            attn_wide_load(regs, Kp, Vt, lo, min(tile + 1, t1 - 1), tid);
            __builtin_amdgcn_sched_barrier(0);
            if (live && tile * 32 < Lw) {                   // uniform over the wave
                uint4 vh[8], vl[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) { vh[k] = buf[1024 + k * 64 + lane]; vl[k] = buf[1536 + k * 64 + lane]; }
                attn_tile(st, vh, vl, qh, ql, buf, tile * 32, qpos, lane);
            }
            __builtin_amdgcn_sched_barrier(0);
            attn_wide_store(regs, attn_lds + (((tile - t0) & 1) ^ 1) * 2048, tid);
            __syncthreads();
        }
    }
    st.lrun += __shfl_xor(st.lrun, 32, 64);
    if (!live) return;

    const size_t unit = ((size_t)task * g.Hkv + kvh) * a.nsplit + split;
    float* po = a.part_o + unit * DH * 32;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r2 = 0; r2 < 16; ++r2) po[(size_t)(dt * 32 + 8 * (r2 >> 2) + 4 * gh + (r2 & 3)) * 32 + i] = st.o[dt][r2];
    if (gh == 0) {
        float* pm = a.part_ml + unit * 64;
        pm[i] = st.mrun; pm[32 + i] = st.lrun;
    }
}

// Merge the key splits of one (task, kv head) and emit the attention output as tiled hi/lo planes
// (K = Hq*128).  grid (tasks * Hkv, 4): workgroup y handles channels 32 y .. 32 y + 31.
__global__ __launch_bounds__(256) void k_chunk_attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                            int nsplit, Geom g, const ChunkTable* __restrict__ tab,
                                                            bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo) {
    constexpr int DH = 128;
    __shared__ float f[CHUNK_ATTN_MAX_SPLIT][32];          // running maximum of every split, then its weight
    __shared__ float fl[CHUNK_ATTN_MAX_SPLIT][32];         // running sum of every split
    __shared__ float red[8][32];
    const int tid = threadIdx.x;
    const int G = g.Hq / g.Hkv;
    const int kvh = blockIdx.x % g.Hkv;
    const ChunkTask T = tab->task[blockIdx.x / g.Hkv];
    const float* ml = part_ml + (size_t)blockIdx.x * nsplit * 64;
    const int j = tid & 31, dl = tid >> 5;                 // column, channel within a run of 8
    const float* po = part_o + (size_t)blockIdx.x * nsplit * DH * 32 + (size_t)(blockIdx.y * 32 + dl) * 32 + j;
    constexpr int PB = 8;                                  // splits whose partial results are requested together
    float p[PB][4];
    auto p_load = [&](int s0) {
#pragma unroll
        for (int k = 0; k < PB; ++k) {
            const int sc = min(s0 + k, nsplit - 1);
#pragma unroll
            for (int u = 0; u < 4; ++u) p[k][u] = po[(size_t)sc * DH * 32 + u * 8 * 32];
        }
    };
    float inv;
    {
        // statistics per query column: thread (column c, slice q) covers splits q, q + 8, ...; partial results meet in
        // LDS.  Maxima and sums of four splits per thread are requested at once, and with the first of them the partial
        // results of the first PB splits, which do not depend on the statistics.
        const int c = tid & 31, q = tid >> 5;
        float m = -INFINITY;
        for (int s0 = q; s0 < nsplit || s0 == q; s0 += 32) {       // every thread runs the first round: it requests p
            float mv[4], lv[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int sc = min(s0 + 8 * k, nsplit - 1);
                mv[k] = ml[sc * 64 + c]; lv[k] = ml[sc * 64 + 32 + c];
            }
            if (s0 == q) p_load(0);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (s0 + 8 * k < nsplit) { f[s0 + 8 * k][c] = mv[k]; fl[s0 + 8 * k][c] = lv[k]; m = fmaxf(m, mv[k]); }
        }
        red[q][c] = m;
        __syncthreads();
        float M = red[0][c];
#pragma unroll
        for (int k = 1; k < 8; ++k) M = fmaxf(M, red[k][c]);
        __syncthreads();
        float lp = 0.f;
        for (int sp = q; sp < nsplit; sp += 8) {
            const float w = f[sp][c] > -INFINITY ? expf(f[sp][c] - M) : 0.f;
            lp += fl[sp][c] * w;
            f[sp][c] = w;
        }
        red[q][c] = lp;
        __syncthreads();
        float L = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) L += red[k][c];
        inv = L > 0.f ? 1.f / L : 0.f;
    }
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; s += PB) {
        if (s > 0) p_load(s);
#pragma unroll
        for (int k = 0; k < PB; ++k) {
            const float w = s + k < nsplit ? f[min(s + k, CHUNK_ATTN_MAX_SPLIT - 1)][j] : 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = fmaf(p[k][u], w, v[u]);
        }
    }
    const int col = 32 * T.tile + j;
    if (col < G * T.n) {
        const int gq = col / T.n, r = col - gq * T.n;
        const int m = T.row0 + r, hq = kvh * G + gq;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ch = blockIdx.y * 32 + dl + 8 * u;
            v[u] *= inv;
            bf16_t hi, lw;
            split_bf16(v[u], hi, lw);
            const size_t o = tiled_off(m, hq * DH + ch, g.Hq * DH);
            out_hi[o] = hi; out_lo[o] = lw;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

hipError_t launch_begin_chunk(const ChunkBuffers& c, const DecodeBuffers& b, int ngroups, hipStream_t s) {
    (void)ngroups;
    hipLaunchKernelGGL(k_begin_chunk, dim3(1), dim3(128), 0, s, c.tab, b.step, b.seq_state, c.chosen);
    return hipGetLastError();
}

hipError_t launch_chunk_embed(const void* E, const ChunkBuffers& c, int rows, const Geom& g, hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_embed, dim3(rows), dim3(256), 0, s, (const bf16_t*)E, c.tab, c.x, g.d);
    return hipGetLastError();
}

static bool row_kernel_ok(const Geom& g, int S) { return g.d % 4 == 0 && g.d <= ROW_VEC_MAX * 1024 && S >= 1 && S <= CHUNK_GEMM_MAX_SPLIT; }

hipError_t launch_chunk_resid_norm(const ChunkBuffers& c, bool add_partials, int S, int MT, const float* gain,
                                   int rows, const Geom& g, hipStream_t s) {
    if (!row_kernel_ok(g, S)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_chunk_resid_norm, dim3(rows), dim3(256), 0, s, c.x, add_partials ? c.part : nullptr, S,
                       (size_t)MT * 32 * g.d, g.d, gain, g.eps, g.d, c.nrm_hi, c.nrm_lo);
    return hipGetLastError();
}

hipError_t launch_chunk_last_row(const ChunkBuffers& c, int S, int MT, int group, const DecodeBuffers& b, const Geom& g,
                                 hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_last_row, dim3((g.d + 255) / 256), dim3(256), 0, s, c.x, c.part, S, (size_t)MT * 32 * g.d,
                       g.d, g.d, c.tab, group, b.step, b.x);
    return hipGetLastError();
}

hipError_t launch_chunk_head_rows(const ChunkBuffers& c, int S, int MT, const float* gain, int ngroups, const Geom& g,
                                  hipStream_t s) {
    if (!row_kernel_ok(g, S)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_chunk_head_rows, dim3(ngroups), dim3(256), 0, s, c.x, c.part, S, (size_t)MT * 32 * g.d, g.d, gain,
                       g.eps, g.d, c.tab, c.nrm_hi, c.nrm_lo);
    return hipGetLastError();
}

hipError_t launch_chunk_logits(const ChunkBuffers& c, int MT_head, float* logits_base, const DecodeBuffers& b, int ngroups,
                               const Geom& g, hipStream_t s) {
    (void)MT_head;
    hipLaunchKernelGGL(k_chunk_logits, dim3(ngroups), dim3(1024), 0, s, c.part, g.V, c.tab, logits_base, b.seq_state, b.banned);
    return hipGetLastError();
}

hipError_t launch_chunk_swiglu(const ChunkBuffers& c, int S, int MT, int rows, const Geom& g, hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_swiglu, dim3((g.F + 255) / 256, rows), dim3(256), 0, s, c.part, S,
                       (size_t)MT * 32 * 2 * g.F, 2 * g.F, g.F, c.act_hi, c.act_lo);
    return hipGetLastError();
}

hipError_t launch_chunk_rope_kv(const ChunkBuffers& c, int S, void* kv_layer, const DecodeBuffers& b, int rows, int MT,
                                const Geom& g, hipStream_t s) {
    const int n_qkv = (g.Hq + 2 * g.Hkv) * g.dh;
    hipLaunchKernelGGL(k_chunk_rope_kv, dim3(g.Hq + 2 * g.Hkv, rows), dim3(g.dh / 2), 0, s, c.part, S, (size_t)MT * 32 * n_qkv,
                       n_qkv, g, c.tab, b.rope_cos, b.rope_sin, (bf16_t*)kv_layer, c.q_hi, c.q_lo, c.q_cols);
    return hipGetLastError();
}

constexpr int ATTN_LDS_BYTES = 4 * 1024 * 16;       // k_chunk_attn: per wave one K tile, two planes

static size_t gemm_lds_bytes(int MT) { return (size_t)(2048 + 2 * MT * 2 * 512) * 16; }
constexpr int GEMM_WIDE_LDS_BYTES = 2 * 2048 * 16;  // k_chunk_gemm_wide: two buffers of one 128 x 128 weight block
// 256-row workgroups of the wide product: four waves with two row tiles each (eight waves with one tile each, two
// per SIMD, measure 2-4 % slower: the loop is bound by operand delivery and power, not by latency)
constexpr int WIDE_NW = 4, WIDE_MW = 2;

hipError_t chunk_init() {
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm<1, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes(1)))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm<1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes(1)))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_attn, hipFuncAttributeMaxDynamicSharedMemorySize, ATTN_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_attn_wide, hipFuncAttributeMaxDynamicSharedMemorySize, ATTN_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_decode_attn_mfma, hipFuncAttributeMaxDynamicSharedMemorySize, ATTN_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_ks<2, false>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_ks<2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_wide<4, 1, false>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_wide<WIDE_NW, WIDE_MW, false>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_wide<4, 1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    if ((e = hipFuncSetAttribute((const void*)k_chunk_gemm_wide<WIDE_NW, WIDE_MW, true>, hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_WIDE_LDS_BYTES))) return e;
    return hipSuccess;
}

hipError_t launch_chunk_gemm(const void* W, int N, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                             int S, int MT, hipStream_t s) {
    const dim3 grid(N / 128, S), block(256);
    const size_t ps = (size_t)MT * 32 * N, lds = gemm_lds_bytes(MT);
    if (S < 1 || S > CHUNK_GEMM_MAX_SPLIT || S > K / 128 || N % 128 || K % 128 || ps * S > c.part_capacity) return hipErrorInvalidValue;
    if (MT < 1 || MT > CHUNK_MAX / 32) return hipErrorInvalidValue;
    // one row tile: weight-streaming kernel, a wave per 32 weight rows; two: the waves split the k-steps; three or four:
    // a wave per row tile (128-row workgroups); more: 256-row workgroups
    if (MT == 1) {
        hipLaunchKernelGGL((k_chunk_gemm<1, false>), grid, block, lds, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S, nullptr, nullptr, 0);
    } else if (MT == 2) {
        hipLaunchKernelGGL((k_chunk_gemm_ks<2, false>), grid, block, GEMM_WIDE_LDS_BYTES, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S, nullptr, nullptr);
    } else {
        const int MY = MT <= 4 ? 1 : (MT + 7) / 8;
        const dim3 wgrid((unsigned)(N / 128) * MY * S);
        if (MT <= 4) hipLaunchKernelGGL((k_chunk_gemm_wide<4, 1, false>), wgrid, block, GEMM_WIDE_LDS_BYTES, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S, MT, nullptr, nullptr);
        else hipLaunchKernelGGL((k_chunk_gemm_wide<WIDE_NW, WIDE_MW, false>), wgrid, dim3(WIDE_NW * 64), GEMM_WIDE_LDS_BYTES, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S, MT, nullptr, nullptr);
    }
    return hipGetLastError();
}

// Gate/up product with the SwiGLU in its epilogue (no split-K): W = [gate rows | up rows] (2F x K), result in
// c.act_hi / c.act_lo.
hipError_t launch_chunk_gemm_swiglu(const void* W, int F, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                                    int MT, hipStream_t s) {
    if (MT < 1 || MT > CHUNK_MAX / 32 || F < 1 || K % 128 || (MT > 1 && F % 64)) return hipErrorInvalidValue;
    const bf16_t* Wb = (const bf16_t*)W;
    if (MT == 1) {
        // gate rows per wave-tile: the fewest whole rounds of tiles over the device's waves that 16 rows per tile allow
        const int waves = 4 * std::max(1, decode_gemv_grid());
        int rp = 16;
        for (int m = 1; m <= 64; ++m) {
            rp = (F + waves * m - 1) / (waves * m);
            if (rp <= 16) break;
        }
        rp = std::min(std::max(rp, 1), 16);
        const int tiles = (F + rp - 1) / rp;
        hipLaunchKernelGGL((k_chunk_gemm<1, true>), dim3((tiles + 3) / 4, 1), dim3(256), gemm_lds_bytes(1), s, Wb, 2 * F, K, xhi, xlo, nullptr, (size_t)0, 0, 1, c.act_hi, c.act_lo, rp);
    } else if (MT == 2) {
        hipLaunchKernelGGL((k_chunk_gemm_ks<2, true>), dim3(F / 64, 1), dim3(256), GEMM_WIDE_LDS_BYTES, s, Wb, 2 * F, K, xhi, xlo, nullptr, (size_t)0, 0, 1, c.act_hi, c.act_lo);
    } else {
        const int MY = MT <= 4 ? 1 : (MT + 7) / 8;
        const dim3 wgrid((unsigned)(F / 64) * MY);
        if (MT <= 4) hipLaunchKernelGGL((k_chunk_gemm_wide<4, 1, true>), wgrid, dim3(256), GEMM_WIDE_LDS_BYTES, s, Wb, 2 * F, K, xhi, xlo, nullptr, (size_t)0, 0, 1, MT, c.act_hi, c.act_lo);
        else hipLaunchKernelGGL((k_chunk_gemm_wide<WIDE_NW, WIDE_MW, true>), wgrid, dim3(WIDE_NW * 64), GEMM_WIDE_LDS_BYTES, s, Wb, 2 * F, K, xhi, xlo, nullptr, (size_t)0, 0, 1, MT, c.act_hi, c.act_lo);
    }
    return hipGetLastError();
}

hipError_t launch_chunk_attn(const ChunkBuffers& c, const void* kv_layer, int nsplit, int ntasks, const Geom& g, hipStream_t s) {
    if (nsplit < 4 || nsplit % 4 || nsplit > CHUNK_ATTN_MAX_SPLIT || ntasks < 1 || ntasks > CHUNK_MAX_TASKS ||
        (long long)ntasks * g.Hkv * nsplit > CHUNK_ATTN_MAX_UNITS)
        return hipErrorInvalidValue;
    ChunkAttnArgs a{};
    a.q_hi = c.q_hi; a.q_lo = c.q_lo; a.kv_layer = (const bf16_t*)kv_layer; a.tab = c.tab;
    a.part_o = c.attn_o; a.part_ml = c.attn_ml; a.nsplit = nsplit; a.q_cols = c.q_cols;
    // one wave per workgroup (the kernel takes any number up to four): the waves of a small pass then spread over more
    // compute units instead of sharing one unit's memory pipeline (24-row inject 4.19 -> 4.11 ms; no change for the
    // 16-sequence batched step)
    hipLaunchKernelGGL(k_chunk_attn, dim3(ntasks * g.Hkv, nsplit), dim3(64), ATTN_LDS_BYTES / 4, s, a, g);
    hipError_t e = hipGetLastError();
    if (e) return e;
    hipLaunchKernelGGL(k_chunk_attn_combine, dim3(ntasks * g.Hkv, 4), dim3(256), 0, s, c.attn_o, c.attn_ml, nsplit, g, c.tab,
                       c.att_hi, c.att_lo);
    return hipGetLastError();
}

// The variant for passes made of large groups: one workgroup per block of up to four tasks, any number of key splits.
hipError_t launch_chunk_attn_wide(const ChunkBuffers& c, const void* kv_layer, int nsplit, int ntasks, int nblocks, const Geom& g,
                                  hipStream_t s) {
    if (nsplit < 1 || nsplit > CHUNK_ATTN_MAX_SPLIT || ntasks < 1 || ntasks > CHUNK_MAX_TASKS || nblocks < 1 || nblocks > ntasks ||
        (long long)ntasks * g.Hkv * nsplit > CHUNK_ATTN_MAX_UNITS)
        return hipErrorInvalidValue;
    ChunkAttnArgs a{};
    a.q_hi = c.q_hi; a.q_lo = c.q_lo; a.kv_layer = (const bf16_t*)kv_layer; a.tab = c.tab;
    a.part_o = c.attn_o; a.part_ml = c.attn_ml; a.nsplit = nsplit; a.q_cols = c.q_cols;
    hipLaunchKernelGGL(k_chunk_attn_wide, dim3(nblocks * g.Hkv, nsplit), dim3(256), ATTN_LDS_BYTES, s, a, g);
    hipError_t e = hipGetLastError();
    if (e) return e;
    hipLaunchKernelGGL(k_chunk_attn_combine, dim3(ntasks * g.Hkv, 4), dim3(256), 0, s, c.attn_o, c.attn_ml, nsplit, g, c.tab,
                       c.att_hi, c.att_lo);
    return hipGetLastError();
}

hipError_t launch_decode_attn_mfma(const ChunkBuffers& c, const void* kv_layer, int nsplit, const DecodeBuffers& b, const Geom& g,
                                   hipStream_t s, unsigned long long* stamps, unsigned long long* done_wg) {
    const int G = g.Hq / g.Hkv;
    if (g.dh != 128 || G > 8 || nsplit < 4 || nsplit % 4 || nsplit > CHUNK_ATTN_MAX_SPLIT ||
        (long long)g.Hkv * nsplit > CHUNK_ATTN_MAX_UNITS)
        return hipErrorInvalidValue;
    DecodeAttnArgs a{};
    a.q = b.q; a.step = b.step; a.kv_layer = (const bf16_t*)kv_layer;
    a.part_o = c.attn_o; a.part_ml = c.attn_ml; a.out = b.o; a.nsplit = nsplit; a.stamps = stamps; a.done_wg = done_wg;
    // one wave per workgroup (the kernel takes any number up to four): the waves that have keys (35 of the 96 splits of a
    // kv head at a context of 1.1k) then spread over as many compute units instead of sharing one unit's memory pipeline
    // four at a time (8B decode 3.31 -> 3.26 ms per token; two per workgroup the same at 1.1k, 2 % slower at 16k)
    hipLaunchKernelGGL(k_decode_attn_mfma, dim3(g.Hkv, nsplit), dim3(64), ATTN_LDS_BYTES / 4, s, a, g);
    hipError_t e = hipGetLastError();
    if (e) return e;
    hipLaunchKernelGGL(k_decode_attn_merge, dim3(g.Hkv, 2 * G), dim3(256), 0, s, a, g);
    return hipGetLastError();
}

}  // namespace asynclm
