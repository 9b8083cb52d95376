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

__global__ void k_begin_chunk(StepDesc* step, SeqState* st, int32_t seq, int32_t rows) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const int32_t len = st[seq].len;
        step->token = -1; step->pos = len; step->seq = seq; step->rows = rows;
        st[seq].len = len + rows;
    }
}

// x[m][:] = E[token_m][:]   (one workgroup per row)
__global__ __launch_bounds__(256) void k_chunk_embed(const bf16_t* __restrict__ E, const int32_t* __restrict__ tokens,
                                                     float* __restrict__ x, int d) {
    const int m = blockIdx.x;
    const bf16_t* row = E + (size_t)tokens[m] * d;
    for (int i = threadIdx.x; i < d; i += 256) x[(size_t)m * d + i] = Elem<bf16_t>::load1(row + i);
}

// x[m] += sum_s P[s][m]  (if P), then RMSNorm with `gain` -> tiled bf16 hi/lo planes.
// One workgroup per row; P has row stride n_stride and split stride s_stride (elements).
__global__ __launch_bounds__(256) void k_chunk_resid_norm(float* __restrict__ x, const float* __restrict__ P, int S,
                                                          size_t s_stride, int n_stride, const float* __restrict__ gain,
                                                          float eps, int d, bf16_t* __restrict__ out_hi,
                                                          bf16_t* __restrict__ out_lo) {
    __shared__ float red[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    float* xr = x + (size_t)m * d;
    float ss = 0.f;
    for (int i = tid; i < d; i += 256) {
        float v = xr[i];
        if (P) {
            for (int s = 0; s < S; ++s) v += P[s * s_stride + (size_t)m * n_stride + i];
            xr[i] = v;
        }
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float sc = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    for (int i = tid; i < d; i += 256) {
        bf16_t hi, lo;
        split_bf16(xr[i] * sc * gain[i], hi, lo);     // xr[i] was written by this same thread
        const size_t o = tiled_off(m, i, d);
        out_hi[o] = hi; out_lo[o] = lo;
    }
}

// Row `row` only: out[:] = x[row] + sum_s P[s][row]  (residual stream handed to the output head)
__global__ __launch_bounds__(256) void k_chunk_last_row(const float* __restrict__ x, const float* __restrict__ P, int S,
                                                        size_t s_stride, int n_stride, int d, const StepDesc* step,
                                                        float* __restrict__ out) {
    const int row = step->rows - 1;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < d; i += gridDim.x * 256) {
        float v = x[(size_t)row * d + i];
        for (int s = 0; s < S; ++s) v += P[s * s_stride + (size_t)row * n_stride + i];
        out[i] = v;
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

// Rotary embedding of q and k, K/V cache write (row-major planes and the transposed V planes),
// scaled q as hi/lo planes [Hq][Mpad][dh].  grid (heads = Hq + 2 Hkv, rows), dh/2 threads.
__global__ void k_chunk_rope_kv(const float* __restrict__ P, int S, size_t s_stride, int n_stride, Geom g,
                                const StepDesc* step, const float* __restrict__ rope_cos,
                                const float* __restrict__ rope_sin, bf16_t* __restrict__ kv_layer,
                                bf16_t* __restrict__ q_hi, bf16_t* __restrict__ q_lo, int Mpad) {
    const int h = blockIdx.x, m = blockIdx.y, i = threadIdx.x, half = g.dh >> 1;
    const int pos = step->pos + m;
    const size_t seq_off = (size_t)step->seq * g.kv_seq_stride;
    float a = 0.f, b = 0.f;
    for (int s = 0; s < S; ++s) {
        const float* p = P + s * s_stride + (size_t)m * n_stride + h * g.dh;
        a += p[i]; b += p[i + half];
    }
    if (h < g.Hq + g.Hkv) {
        const float c = rope_cos[(size_t)pos * half + i], sn = rope_sin[(size_t)pos * half + i];
        const float ra = a * c - b * sn, rb = b * c + a * sn;
        a = ra; b = rb;
    }
    bf16_t ahi, alo, bhi, blo;
    if (h < g.Hq) {
        split_bf16(a * g.scale, ahi, alo); split_bf16(b * g.scale, bhi, blo);
        const size_t o = ((size_t)h * Mpad + m) * g.dh;
        q_hi[o + i] = ahi; q_lo[o + i] = alo; q_hi[o + i + half] = bhi; q_lo[o + i + half] = blo;
        return;
    }
    split_bf16(a, ahi, alo); split_bf16(b, bhi, blo);
    if (h < g.Hq + g.Hkv) {
        bf16_t* kp = kv_layer + seq_off + (size_t)(h - g.Hq) * g.kv_head_stride + (size_t)pos * g.dh;
        kp[i] = ahi; kp[i + half] = bhi; kp[g.kv_lo_offset + i] = alo; kp[g.kv_lo_offset + i + half] = blo;
    } else {
        const int vh = h - g.Hq - g.Hkv;
        bf16_t* vp = kv_layer + g.kv_v_offset + seq_off + (size_t)vh * g.kv_head_stride + (size_t)pos * g.dh;
        vp[i] = ahi; vp[i + half] = bhi; vp[g.kv_lo_offset + i] = alo; vp[g.kv_lo_offset + i + half] = blo;
        bf16_t* vt = kv_layer + g.kv_vt_offset + seq_off + (size_t)vh * g.kv_head_stride + pos;   // [dh][max_pos]
        vt[(size_t)i * g.max_pos] = ahi; vt[(size_t)(i + half) * g.max_pos] = bhi;
        vt[g.kv_lo_offset + (size_t)i * g.max_pos] = alo; vt[g.kv_lo_offset + (size_t)(i + half) * g.max_pos] = blo;
    }
}

// ---------------------------------------------------------------------------------------------
// skinny GEMM on the matrix cores:  P[s][m][n] = sum_{k in slice} X[m][k] W[n][k]
// ---------------------------------------------------------------------------------------------
// Workgroup = 4 waves on the same 32 weight rows; the 4*S waves of a row tile split K into
// contiguous runs of 128-element blocks.  A wave keeps the whole 32 x Mpad accumulator; the four
// partial accumulators of a workgroup are summed through LDS, the S workgroups of a row tile
// write separate partial planes that the consumer adds in a fixed order (no atomics).

// Operands of one 128-element k-block for one wave: 32 weight rows x 128 as loaded (4 rows per
// instruction: lane l holds row 4q + l/16, 16-byte chunk l%16) and Mpad token rows x 128 in operand order.
template <int MT>
struct GemmTile {
    uint4 a[8];
    uint4 bh[MT][8], bl[MT][8];
};

template <int MT>
__device__ __forceinline__ void gemm_tile_load(GemmTile<MT>& t, const bf16_t* wlane, size_t wstep, const bf16_t* const (&xh)[MT],
                                               const bf16_t* const (&xl)[MT], int blk) {
#pragma unroll
    for (int q = 0; q < 8; ++q) t.a[q] = load16_stream(wlane + (size_t)blk * 128 + q * wstep);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            t.bh[mt][k] = load16(xh[mt] + (size_t)blk * 4096 + k * 512);
            t.bl[mt][k] = load16(xl[mt] + (size_t)blk * 4096 + k * 512);
        }
}

// Transposes the weight tile into operand order through the wave's LDS tile, then multiplies.
// LDS tile: 32 rows x 16 chunks of 16 bytes, chunk c of row r stored at chunk position c ^ (r & 15).
template <int MT>
__device__ __forceinline__ void gemm_tile_mma(const GemmTile<MT>& t, f32x16 (&acc)[MT], uint4* lds, int lane) {
    {
        const int r0 = lane >> 4, c = lane & 15;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int r = 4 * q + r0;
            lds[r * 16 + (c ^ (r & 15))] = t.a[q];
        }
    }
    uint4 a[8];
    {
        const int i = lane & 31, gh = lane >> 5;
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] = lds[i * 16 + ((2 * k + gh) ^ (i & 15))];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = mfma_bf16(a[k], t.bh[mt][k], acc[mt]);
            acc[mt] = mfma_bf16(a[k], t.bl[mt][k], acc[mt]);
        }
}

template <int MT>
__global__ __launch_bounds__(256) void k_chunk_gemm(const bf16_t* __restrict__ W, int N, int K,
                                                    const bf16_t* __restrict__ Xhi, const bf16_t* __restrict__ Xlo,
                                                    float* __restrict__ P, size_t s_stride, int n_stride, int S) {
    // per-wave weight tiles (8 KiB each) during the product, then the four partial accumulators
    constexpr int RED_BYTES = 4 * MT * 16 * 64 * 4, LDS_BYTES = RED_BYTES > 32768 ? RED_BYTES : 32768;
    __shared__ uint4 lds_raw[LDS_BYTES / 16];
    uint4 (*wt)[512] = reinterpret_cast<uint4 (*)[512]>(lds_raw);
    float (*red)[MT][16][64] = reinterpret_cast<float (*)[MT][16][64]>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * 32, sp = blockIdx.y;
    // K is split over the 4*S waves of this row tile in units of two 128-element blocks
    const int npair = K >> 8, parts = 4 * S, part = sp * 4 + wave;
    const int b0 = 2 * (int)((long long)npair * part / parts), b1 = 2 * (int)((long long)npair * (part + 1) / parts);

    const bf16_t* wlane = W + (size_t)(n0 + (lane >> 4)) * K + (lane & 15) * 8;   // row l/16 (+4q), chunk l%16
    const size_t wstep = (size_t)4 * K;
    const bf16_t* xh[MT]; const bf16_t* xl[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        xh[mt] = Xhi + (size_t)mt * 32 * K + lane * 8;
        xl[mt] = Xlo + (size_t)mt * 32 * K + lane * 8;
    }
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

    // Two register tiles in ping-pong over pairs of k-blocks: the loads of the next block are in flight
    // while the current one is multiplied.  The body has no conditional code (a wave always owns an even
    // number of blocks; past its end it re-reads its last block and drops it), because the compiler sinks
    // loads into conditional users and then waits for each load right before its product.  The scheduling
    // barriers keep the instruction scheduler from doing the same within the straight-line body.
    GemmTile<MT> t0, t1;
    if (b0 < b1) {
        gemm_tile_load<MT>(t0, wlane, wstep, xh, xl, b0);
        for (int b = b0; b < b1; b += 2) {
            gemm_tile_load<MT>(t1, wlane, wstep, xh, xl, b + 1);
            __builtin_amdgcn_sched_barrier(0);
            gemm_tile_mma<MT>(t0, acc, wt[wave], lane);
            __builtin_amdgcn_sched_barrier(0);
            gemm_tile_load<MT>(t0, wlane, wstep, xh, xl, min(b + 2, b1 - 1));
            __builtin_amdgcn_sched_barrier(0);
            gemm_tile_mma<MT>(t1, acc, wt[wave], lane);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    __syncthreads();        // every wave is done with its weight tile
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][mt][r][lane] = acc[mt][r];
    __syncthreads();
    // thread -> (token column j, four consecutive weight rows): coalesced 16-byte stores
    const int j = tid >> 3, q = tid & 7, b = q >> 1, g2 = q & 1;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float4 v;
        float* vp = &v.x;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int idx = 4 * b + r, ln = j + 32 * g2;
            vp[r] = red[0][mt][idx][ln] + red[1][mt][idx][ln] + red[2][mt][idx][ln] + red[3][mt][idx][ln];
        }
        *(float4*)(P + sp * s_stride + (size_t)(mt * 32 + j) * n_stride + n0 + 4 * q) = v;
    }
}

// ---------------------------------------------------------------------------------------------
// causal chunk attention on the matrix cores (head_dim 128, paired bf16 cache)
// ---------------------------------------------------------------------------------------------
// One wave = one (kv head, tile of 32 query rows, key split).  Query rows of a kv head are ordered
// [q head within the group][row m], padded to Mpad rows per head.  Per 32-key tile the wave forms
// S^T = K Q^T (keys along D rows), does the online softmax per query column, and accumulates
// O^T += V^T P^T from the transposed V planes.  Key rows are permuted so that the D registers of a
// lane hold 16 consecutive keys, which makes P directly usable as the next B operand.

struct ChunkAttnArgs {
    const bf16_t* q_hi; const bf16_t* q_lo;     // [Hq][Mpad][128], scaled by 1/sqrt(dh)
    const bf16_t* kv_layer;
    const StepDesc* step;
    float* part_o;      // [task][split][128][32]
    float* part_ml;     // [task][split][2][32]
    int32_t nsplit, MT;
};

__global__ __launch_bounds__(256) void k_chunk_attn(ChunkAttnArgs a, Geom g) {
    constexpr int DH = 128;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, gh = lane >> 5;
    const int G = g.Hq / g.Hkv;
    const int task = blockIdx.x, split = blockIdx.y * 4 + wave;
    const int tiles_q = G * a.MT;
    const int kvh = task / tiles_q, qt = task - kvh * tiles_q;
    const int hq = kvh * G + qt / a.MT, m0 = (qt % a.MT) * 32;
    const int Mpad = a.MT * 32;
    const int pos0 = a.step->pos, rows = a.step->rows;
    const int Lk = pos0 + rows;                           // keys 0 .. Lk-1 exist
    const int ntile = (Lk + 31) >> 5;
    const int tps = (ntile + a.nsplit - 1) / a.nsplit;
    const int t0 = split * tps, t1 = min(ntile, t0 + tps);

    const size_t seq_off = (size_t)a.step->seq * g.kv_seq_stride + (size_t)kvh * g.kv_head_stride;
    const bf16_t* Kp = a.kv_layer + seq_off;
    const bf16_t* Vt = a.kv_layer + g.kv_vt_offset + seq_off;
    const size_t lo = g.kv_lo_offset;

    // B operand of S^T = K Q^T: lane (j, g) holds q[j][64 g + 8 t + e]
    uint4 qh[8], ql[8];
    {
        const bf16_t* qp = a.q_hi + ((size_t)hq * Mpad + m0 + i) * DH + gh * 64;
        const bf16_t* qq = a.q_lo + ((size_t)hq * Mpad + m0 + i) * DH + gh * 64;
#pragma unroll
        for (int t = 0; t < 8; ++t) { qh[t] = load16(qp + t * 8); ql[t] = load16(qq + t * 8); }
    }
    const int qpos = pos0 + m0 + i;                        // position of this lane's query column
    const int krow = (i >> 3) * 4 + (i & 3) + 16 * ((i >> 2) & 1);   // key (within a tile) held in A row i

    f32x16 o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;

    for (int tile = t0; tile < t1; ++tile) {
        const int key0 = tile * 32;
        if (key0 > pos0 + m0 + 31) break;                   // beyond the causal limit of every row
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        {
            const bf16_t* kp = Kp + (size_t)(key0 + krow) * DH + gh * 64;
            uint4 kh[8], kl[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) { kh[t] = load16(kp + t * 8); kl[t] = load16(kp + lo + t * 8); }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                s = mfma_bf16(kh[t], qh[t], s);
                s = mfma_bf16(kl[t], qh[t], s);
                s = mfma_bf16(kh[t], ql[t], s);
            }
        }
        // register r of lane (j, g) is key key0 + 16 g + r for query column j
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (key0 + 16 * gh + r > qpos) s[r] = -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mnew = fmaxf(mrun, mx);
        const float msafe = mnew == -INFINITY ? 0.f : mnew;
        const float corr = expf(mrun - msafe);
        float psum = 0.f;
        uint4 ph[2], pl[2];
        {
            bf16_t hi[16], lw[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = expf(s[r] - msafe);
                psum += p;
                split_bf16(p, hi[r], lw[r]);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                ph[t] = make_uint4(hi[8 * t] | ((uint32_t)hi[8 * t + 1] << 16), hi[8 * t + 2] | ((uint32_t)hi[8 * t + 3] << 16),
                                   hi[8 * t + 4] | ((uint32_t)hi[8 * t + 5] << 16), hi[8 * t + 6] | ((uint32_t)hi[8 * t + 7] << 16));
                pl[t] = make_uint4(lw[8 * t] | ((uint32_t)lw[8 * t + 1] << 16), lw[8 * t + 2] | ((uint32_t)lw[8 * t + 3] << 16),
                                   lw[8 * t + 4] | ((uint32_t)lw[8 * t + 5] << 16), lw[8 * t + 6] | ((uint32_t)lw[8 * t + 7] << 16));
            }
        }
        lrun = lrun * corr + psum;
        mrun = mnew;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= corr;
            const bf16_t* vp = Vt + (size_t)(dt * 32 + i) * g.max_pos + key0 + 16 * gh;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint4 vh = load16(vp + 8 * t), vl = load16(vp + lo + 8 * t);
                o[dt] = mfma_bf16(vh, ph[t], o[dt]);
                o[dt] = mfma_bf16(vl, ph[t], o[dt]);
                o[dt] = mfma_bf16(vh, pl[t], o[dt]);
            }
        }
    }
    lrun += __shfl_xor(lrun, 32, 64);

    float* po = a.part_o + ((size_t)task * a.nsplit + split) * DH * 32;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) po[(size_t)(dt * 32 + 8 * (r >> 2) + 4 * gh + (r & 3)) * 32 + i] = o[dt][r];
    if (gh == 0) {
        float* pm = a.part_ml + ((size_t)task * a.nsplit + split) * 64;
        pm[i] = mrun; pm[32 + i] = lrun;
    }
}

// Merge the key splits of one task and emit the attention output as tiled hi/lo planes (K = Hq*128).
__global__ __launch_bounds__(256) void k_chunk_attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                            int nsplit, int MT, Geom g, const StepDesc* step,
                                                            bf16_t* __restrict__ out_hi, bf16_t* __restrict__ out_lo) {
    constexpr int DH = 128;
    __shared__ float f[ATTN_MAX_SPLIT][32];
    const int task = blockIdx.x, tid = threadIdx.x;
    const int G = g.Hq / g.Hkv, tiles_q = G * MT;
    const int kvh = task / tiles_q, qt = task - kvh * tiles_q;
    const int hq = kvh * G + qt / MT, m0 = (qt % MT) * 32;
    const float* ml = part_ml + (size_t)task * nsplit * 64;
    if (tid < 32) {
        float M = -INFINITY, L = 0.f;
        for (int s = 0; s < nsplit; ++s) M = fmaxf(M, ml[s * 64 + tid]);
        for (int s = 0; s < nsplit; ++s) {
            const float ms = ml[s * 64 + tid];
            const float w = ms > -INFINITY ? expf(ms - M) : 0.f;
            L += ml[s * 64 + 32 + tid] * w;
            f[s][tid] = w;
        }
        const float inv = L > 0.f ? 1.f / L : 0.f;
        for (int s = 0; s < nsplit; ++s) f[s][tid] *= inv;
    }
    __syncthreads();
    const int rows = step->rows;
    const float* po = part_o + (size_t)task * nsplit * DH * 32;
    for (int e = tid; e < DH * 32; e += 256) {
        const int dh = e >> 5, j = e & 31;
        float v = 0.f;
#pragma unroll 4
        for (int s = 0; s < nsplit; ++s) v = fmaf(po[(size_t)s * DH * 32 + e], f[s][j], v);
        const int m = m0 + j;
        if (m < rows) {
            bf16_t hi, lw;
            split_bf16(v, hi, lw);
            const size_t o = tiled_off(m, hq * DH + dh, g.Hq * DH);
            out_hi[o] = hi; out_lo[o] = lw;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

hipError_t launch_begin_chunk(const DecodeBuffers& b, int seq, int rows, hipStream_t s) {
    hipLaunchKernelGGL(k_begin_chunk, dim3(1), dim3(64), 0, s, b.step, b.seq_state, seq, rows);
    return hipGetLastError();
}

hipError_t launch_chunk_embed(const void* E, const ChunkBuffers& c, int rows, const Geom& g, hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_embed, dim3(rows), dim3(256), 0, s, (const bf16_t*)E, c.tokens, c.x, g.d);
    return hipGetLastError();
}

hipError_t launch_chunk_resid_norm(const ChunkBuffers& c, bool add_partials, int S, int MT, const float* gain,
                                   int rows, const Geom& g, hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_resid_norm, dim3(rows), dim3(256), 0, s, c.x, add_partials ? c.part : nullptr, S,
                       (size_t)MT * 32 * g.d, g.d, gain, g.eps, g.d, c.nrm_hi, c.nrm_lo);
    return hipGetLastError();
}

hipError_t launch_chunk_last_row(const ChunkBuffers& c, int S, int MT, const DecodeBuffers& b, const Geom& g,
                                 hipStream_t s) {
    hipLaunchKernelGGL(k_chunk_last_row, dim3((g.d + 255) / 256), dim3(256), 0, s, c.x, c.part, S, (size_t)MT * 32 * g.d,
                       g.d, g.d, b.step, b.x);
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
                       n_qkv, g, b.step, b.rope_cos, b.rope_sin, (bf16_t*)kv_layer, c.q_hi, c.q_lo,
                       MT * 32);
    return hipGetLastError();
}

hipError_t launch_chunk_gemm(const void* W, int N, int K, const bf16_t* xhi, const bf16_t* xlo, const ChunkBuffers& c,
                             int S, int MT, hipStream_t s) {
    const dim3 grid(N / 32, S), block(256);
    const size_t ps = (size_t)MT * 32 * N;
    if (S < 1 || S > CHUNK_GEMM_MAX_SPLIT || N % 32 || K % 256 || ps * S > c.part_capacity) return hipErrorInvalidValue;
    if (MT == 1) hipLaunchKernelGGL(k_chunk_gemm<1>, grid, block, 0, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S);
    else if (MT == 2) hipLaunchKernelGGL(k_chunk_gemm<2>, grid, block, 0, s, (const bf16_t*)W, N, K, xhi, xlo, c.part, ps, N, S);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_chunk_attn(const ChunkBuffers& c, const void* kv_layer, int nsplit, int MT, const DecodeBuffers& b,
                             const Geom& g, hipStream_t s) {
    ChunkAttnArgs a{};
    a.q_hi = c.q_hi; a.q_lo = c.q_lo; a.kv_layer = (const bf16_t*)kv_layer; a.step = b.step;
    a.part_o = c.attn_o; a.part_ml = c.attn_ml; a.nsplit = nsplit; a.MT = MT;
    const int tasks = g.Hkv * (g.Hq / g.Hkv) * MT;
    hipLaunchKernelGGL(k_chunk_attn, dim3(tasks, nsplit / 4), dim3(256), 0, s, a, g);
    hipError_t e = hipGetLastError();
    if (e) return e;
    hipLaunchKernelGGL(k_chunk_attn_combine, dim3(tasks), dim3(256), 0, s, c.attn_o, c.attn_ml, nsplit, MT, g, b.step,
                       c.att_hi, c.att_lo);
    return hipGetLastError();
}

}  // namespace asynclm
