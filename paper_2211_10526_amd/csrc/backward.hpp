// Backward pass of the layer on the vector ALU (any I/O type, fp32 arithmetic): the gradients of
// Eq. 3 / 8 / 9 with respect to q, k, v, the DWConv filters and their bias, given g = dLoss/dout.
//
// With num_t = vsum / 2 + q_hat_t S / pi and den_t = N / 2 + q_hat_t . ksum / pi (Eq. 3 after the
// reassociation of Sec. 3.1), a_t = dLoss/dnum_t = g_t / den_t and
// b_t = dLoss/dden_t = -(g_t . lin_t) / den_t  (a_t = g_t, b_t = 0 without the normaliser):
//   dq_hat_t = (S a_t + ksum b_t) / pi
//   S' = sum_t q_hat_t^T a_t,   kb' = sum_t q_hat_t b_t,   va' = sum_t a_t
//   dv_j     = k_hat_j S' / pi + va' / 2 + (DWConv of g with the filters turned by 180 degrees)
//   dk_hat_j = (S' v_j + kb') / pi
//   dx = (dx_hat - x_hat (x_hat . dx_hat)) / |x|   (dx_hat / eps where |x| < eps)
// S', va' are what pass 1 computes from (q, a) in place of (k, v), and dv is what pass 2 computes
// from (k, g) with that state: both reuse the forward kernels.  This file holds the rest: the
// per-row kernel (a, b, dq; dk), the filter gradient and small helpers.
#pragma once

#include "apply_generic.hpp"
#include "common.hpp"

namespace castling {

struct BwdRowsParams {
    int N;           // tokens per unit
    int tiles;       // ceil(N / 64)
    int norm_none;
    int residual_q;  // QUERY: dq gains g
    int d_valid;     // features per head in memory (<= D)
    float eps;
    // a is stored times ascale (N with the normaliser: a_t = g_t / den_t is of the order g / N,
    // below the normal range of fp16 for long sequences; 1 without), so the state of (q, a) is
    // ascale times S', va'.  mscale: factor on the state matrix as it is loaded (1/pi for the
    // forward state, 1/(pi ascale) for the state of (q, a)).
    float ascale, mscale;
    TensorStrides in, out;  // of q, k, v, a and the gradients of q, k; of g
};

// R consecutive elements at p (R * sizeof(T) a power of two; p aligned to min(that, 16) bytes)
// as one access, widened to fp32 / narrowed from it.
template <typename T, int R>
__device__ __forceinline__ void load_piece(const T* p, float (&x)[R])
{
    constexpr int BYTES = sizeof(T) * R;
    __attribute__((aligned(16))) T tmp[R];
    if constexpr (BYTES % 16 == 0) {
#pragma unroll
        for (int c = 0; c < BYTES / 16; ++c)
            reinterpret_cast<uint4*>(tmp)[c] = reinterpret_cast<const uint4*>(p)[c];
    } else if constexpr (BYTES == 8) {
        *reinterpret_cast<uint2*>(tmp) = *reinterpret_cast<const uint2*>(p);
    } else if constexpr (BYTES == 4) {
        *reinterpret_cast<uint32_t*>(tmp) = *reinterpret_cast<const uint32_t*>(p);
    } else {
        static_assert(BYTES == 2, "piece of one thread");
        tmp[0] = *p;
    }
#pragma unroll
    for (int j = 0; j < R; ++j) x[j] = IO<T>::to_f32(tmp[j]);
}

template <typename T, int R>
__device__ __forceinline__ void store_piece(T* p, const float (&x)[R])
{
    constexpr int BYTES = sizeof(T) * R;
    __attribute__((aligned(16))) T tmp[R];
#pragma unroll
    for (int j = 0; j < R; ++j) tmp[j] = IO<T>::from_f32(x[j]);
    if constexpr (BYTES % 16 == 0) {
#pragma unroll
        for (int c = 0; c < BYTES / 16; ++c)
            reinterpret_cast<uint4*>(p)[c] = reinterpret_cast<const uint4*>(tmp)[c];
    } else if constexpr (BYTES == 8) {
        *reinterpret_cast<uint2*>(p) = *reinterpret_cast<const uint2*>(tmp);
    } else if constexpr (BYTES == 4) {
        *reinterpret_cast<uint32_t*>(p) = *reinterpret_cast<const uint32_t*>(tmp);
    } else {
        static_assert(BYTES == 2, "piece of one thread");
        *p = tmp[0];
    }
}

constexpr int kBwdTokens = 64;             // tokens per block
constexpr int kBwdTStride = kBwdTokens + 4;  // floats; keeps float4 rows aligned

template <int D>
constexpr size_t bwd_rows_lds_bytes()
{
    // M [D][D+1], vec [D], vs [D], xt [D][68], at [D][68], inv / small / b [64] each
    return sizeof(float) * (static_cast<size_t>(D) * (D + 1) + 2 * D + 2 * D * kBwdTStride + 3 * kBwdTokens);
}

// grid = (ceil(N / 64), units), block = 256, dynamic LDS = bwd_rows_lds_bytes<D>().
// QUERY: x = q.  Recomputes num, den of the unit's tokens from `state` (the forward state),
//   writes a (type T, layout of q) to `a_out`, this tile's share of kb' to
//   kb_part[unit][tile][D], and dq to `dx`.
// !QUERY: x = k, `y` = v, `state` = (S', -, -) and `vec` = kb' of the unit ([units][D]): writes dk.
// Thread (tt, tj) = (tid / 16, tid % 16) owns tokens 4 tt .. 4 tt + 3 and features tj D/16 .. .
template <typename T, int D, bool QUERY>
__global__ __launch_bounds__(256) void bwd_rows_kernel(const T* __restrict__ x,
                                                       const T* __restrict__ y,
                                                       const float* __restrict__ state,
                                                       const float* __restrict__ vec,
                                                       T* __restrict__ a_out,
                                                       float* __restrict__ kb_part,
                                                       T* __restrict__ dx, int heads, BwdRowsParams p)
{
    constexpr int VEC = IO<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int RJ = D / 16;
    constexpr int MS = D + 1;  // row stride of M: the second product walks its columns
    using L = StateLayout<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    float* M = reinterpret_cast<float*>(lds_raw);
    float* vk = M + D * MS;             // ksum / pi   (kb' / pi)
    float* vs = vk + D;                 // vsum / 2
    float* xt = vs + D;                 // unit rows of x, transposed [D][68]
    float* at = xt + D * kBwdTStride;   // a (or v), transposed [D][68]
    float* inv = at + D * kBwdTStride;  // 1 / max(|x|, eps)
    float* small = inv + kBwdTokens;    // 1 where |x| < eps
    float* bs = small + kBwdTokens;     // b_t

    const int tid = threadIdx.x;
    const int unit = blockIdx.y, tile = blockIdx.x;
    const int n0 = tile * kBwdTokens;
    const int tt = tid / 16, tj = tid % 16;
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long out_off = unit_offset(unit, heads, p.out);

    const float* gs = state + static_cast<size_t>(unit) * L::SIZE;
    block_stage<D * D, float>(
        tid, [&](int i) { return gs[L::S + i]; },
        [&](int i, float s) { M[(i / D) * MS + i % D] = s * p.mscale; });
    if (tid < D) {
        vk[tid] = (QUERY ? gs[L::KSUM + tid] : vec[static_cast<size_t>(unit) * D + tid]) * kInvPi;
        vs[tid] = 0.5f * gs[L::VSUM + tid];
    }

    // rows of x -> unit rows, transposed; !QUERY: rows of y (= v) -> at
    constexpr int ROWS = 256 / LPR;
    constexpr int PASSES = (kBwdTokens + ROWS - 1) / ROWS;
    const int lcol = (tid % LPR) * VEC;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
        const int tl = pass * ROWS + tid / LPR;
        if (tl >= kBwdTokens) break;
        const int n = n0 + tl;
        float xv[VEC], yv[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) xv[e] = yv[e] = 0.f;
        if (n < p.N && lcol < p.d_valid) {
            IO<T>::load16(x + in_off + n * p.in.n + lcol, xv);
            if (!QUERY) IO<T>::load16(y + in_off + n * p.in.n + lcol, yv);
        }
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) ss += xv[e] * xv[e];
        ss = group_sum<LPR>(ss);
        const float nrm = sqrtf(ss);
        const float r = 1.0f / fmaxf(nrm, p.eps);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            xt[(lcol + e) * kBwdTStride + tl] = xv[e] * r;
            if (!QUERY) at[(lcol + e) * kBwdTStride + tl] = yv[e];
        }
        if (tid % LPR == 0) {
            inv[tl] = r;
            small[tl] = nrm < p.eps ? 1.f : 0.f;
            if (!QUERY) bs[tl] = 1.f;
        }
    }
    __syncthreads();

    float gown[4][RJ] = {};  // QUERY: g of the own tokens and features (for the residual)
    if (QUERY) {
        // forward quantities of the own tokens: num (own features), den
        float num[4][RJ], den[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < RJ; ++j) num[t][j] = 0.f;
#pragma unroll 4
        for (int i = 0; i < D; ++i) {
            const float4 x4 = *reinterpret_cast<const float4*>(xt + i * kBwdTStride + tt * 4);
            const float xa[4] = {x4.x, x4.y, x4.z, x4.w};
            const float ki = vk[i];
            float m[RJ];
#pragma unroll
            for (int j = 0; j < RJ; ++j) m[j] = M[i * MS + tj * RJ + j];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                den[t] = fmaf(xa[t], ki, den[t]);
#pragma unroll
                for (int j = 0; j < RJ; ++j) num[t][j] = fmaf(xa[t], m[j], num[t][j]);
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int n = n0 + tt * 4 + t;
            const bool live = n < p.N && tj * RJ < p.d_valid;
            if (live) load_piece<T, RJ>(y + out_off + n * p.out.n + tj * RJ, gown[t]);  // y = g
            float gl = 0.f;
            const float rden = 1.0f / (0.5f * static_cast<float>(p.N) + den[t]);
#pragma unroll
            for (int j = 0; j < RJ; ++j)
                gl = fmaf(gown[t][j], (vs[tj * RJ + j] + num[t][j]) * rden, gl);
            gl = group_sum<16>(gl);  // g_t . lin_t over all features
            const float bt = p.norm_none ? 0.f : -gl * rden;
            float av[RJ];
#pragma unroll
            for (int j = 0; j < RJ; ++j) {
                const float a0 = p.norm_none ? gown[t][j] : gown[t][j] * rden;
                at[(tj * RJ + j) * kBwdTStride + tt * 4 + t] = a0;
                av[j] = a0 * p.ascale;
            }
            if (live) store_piece<T, RJ>(a_out + in_off + n * p.in.n + tj * RJ, av);
            if (tj == 0) bs[tt * 4 + t] = n < p.N ? bt : 0.f;
        }
        __syncthreads();
        // this tile's share of kb' = sum_t q_hat_t b_t
        if (tid < D) {
            float s = 0.f;
#pragma unroll 8
            for (int t = 0; t < kBwdTokens; ++t) s = fmaf(xt[tid * kBwdTStride + t], bs[t], s);
            kb_part[(static_cast<size_t>(unit) * p.tiles + tile) * D + tid] = s;
        }
    }

    // dx_hat (own tokens, own features i) = sum_c M[i][c] at[c][t] + vk[i] b_t
    float dxh[4][RJ];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < RJ; ++j) dxh[t][j] = vk[tj * RJ + j] * bs[tt * 4 + t];
#pragma unroll 4
    for (int c = 0; c < D; ++c) {
        const float4 a4 = *reinterpret_cast<const float4*>(at + c * kBwdTStride + tt * 4);
        const float aa[4] = {a4.x, a4.y, a4.z, a4.w};
        float m[RJ];
#pragma unroll
        for (int j = 0; j < RJ; ++j) m[j] = M[(tj * RJ + j) * MS + c];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < RJ; ++j) dxh[t][j] = fmaf(aa[t], m[j], dxh[t][j]);
    }
    // back through the normalisation, store
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int tl = tt * 4 + t, n = n0 + tl;
        float xh[RJ], dot = 0.f;
#pragma unroll
        for (int j = 0; j < RJ; ++j) {
            xh[j] = xt[(tj * RJ + j) * kBwdTStride + tl];
            dot = fmaf(xh[j], dxh[t][j], dot);
        }
        dot = group_sum<16>(dot);
        if (small[tl] != 0.f) dot = 0.f;  // below the floor the row is x / eps: no projection
        if (n < p.N && tj * RJ < p.d_valid) {
            float r[RJ];
#pragma unroll
            for (int j = 0; j < RJ; ++j) {
                r[j] = (dxh[t][j] - xh[j] * dot) * inv[tl];
                if (QUERY && p.residual_q) r[j] += gown[t][j];
            }
            store_piece<T, RJ>(dx + in_off + n * p.in.n + tj * RJ, r);
        }
    }
}

// grid = (units), block = 128: kb[unit][i] = sum over tiles of kb_part[unit][tile][i], in order.
__global__ __launch_bounds__(128) void bwd_vec_combine_kernel(const float* __restrict__ kb_part,
                                                              float* __restrict__ kb, int tiles, int D)
{
    const int i = threadIdx.x;
    if (i >= D) return;
    const float* src = kb_part + static_cast<size_t>(blockIdx.x) * tiles * D + i;
    kb[static_cast<size_t>(blockIdx.x) * D + i] = sum_partials(src, tiles, D);
}

// grid = (ceil(n / 256)), block = 256: the filters [heads * d][ks][ks] turned by 180 degrees.
template <typename T>
__global__ __launch_bounds__(256) void flip_filters_kernel(const T* __restrict__ w, T* __restrict__ out,
                                                           int n, int taps)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int ch = i / taps, e = i % taps;
    out[i] = w[ch * taps + (taps - 1 - e)];
}

// grid = (ceil(n / 256)), block = 256
__global__ __launch_bounds__(256) void fill_zero_f32_kernel(float* __restrict__ p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

struct BwdFilterParams {
    int grid_h, grid_w;
    int tiles_x, n_tiles;  // 4 x 16 tiles of the grid
    int chunks;            // blocks per unit; block c takes tiles c, c + chunks, ...
    int d_valid;
    TensorStrides in, out;  // of v; of g
};

template <typename T, int D, int KS>
constexpr size_t bwd_filter_lds_bytes()
{
    return sizeof(T) * ((kApplyTH + KS - 1) * (kApplyTW + KS - 1) + kApplyTokens) * D;
}

// Filter and bias gradients: dw[c][dy][dx] = sum over tokens of g[t][c] v[t + (dy, dx) - r][c],
// dbias[c] = sum of g[t][c].  grid = (chunks, units), block = 256, dynamic LDS =
// bwd_filter_lds_bytes.  Thread (part, c) = (tid / (D/2), 2 (tid % (D/2))) accumulates the taps
// part, part + 512 / D, ... of channels c, c + 1 over the block's tiles (and the sum of g, the
// bias gradient, as tap KS * KS) and writes them to part_out[unit][chunk][tap][D]; v, g point
// at the first grid token.
template <typename T>
struct alignas(2 * sizeof(T)) ChannelPair {
    T a, b;
};

template <typename T, int D, int KS>
__global__ __launch_bounds__(256) void bwd_filter_kernel(const T* __restrict__ v,
                                                         const T* __restrict__ g,
                                                         float* __restrict__ part_out, int heads,
                                                         BwdFilterParams p)
{
    constexpr int VEC = IO<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int RAD = KS / 2;
    constexpr int HH = kApplyTH + KS - 1, HW = kApplyTW + KS - 1;
    using Pair = ChannelPair<T>;
    constexpr int TPC = 512 / D;                     // threads per pair of channels
    constexpr int NT = KS * KS + 1;                  // taps and the bias
    constexpr int TAPS = (KS * KS + TPC - 1) / TPC;  // per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T* vh = reinterpret_cast<T*>(lds_raw);  // [HH][HW][D], zero outside the grid
    T* gt = vh + HH * HW * D;               // [4 x 16 tokens][D], zero outside the grid

    const int tid = threadIdx.x;
    const int unit = blockIdx.y;
    const int c = 2 * (tid % (D / 2)), part = tid / (D / 2);
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long out_off = unit_offset(unit, heads, p.out);

    // LDS element offset of the thread's taps relative to a token (taps past the last one read
    // tap 0 and are dropped at the end)
    int tap_off[TAPS];
#pragma unroll
    for (int i = 0; i < TAPS; ++i) {
        const int e = part + TPC * i;
        tap_off[i] = e < KS * KS ? ((e / KS) * HW + e % KS) * D : 0;
    }
    float acc[TAPS][2], gsum[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < TAPS; ++i) acc[i][0] = acc[i][1] = 0.f;

    for (int tile = blockIdx.x; tile < p.n_tiles; tile += p.chunks) {
        const int ty0 = (tile / p.tiles_x) * kApplyTH, tx0 = (tile % p.tiles_x) * kApplyTW;
        __syncthreads();  // the previous tile's reads are done
        for (int idx = tid; idx < HH * HW * LPR; idx += 256) {
            const int tok = idx / LPR, piece = idx % LPR;
            const int yy = ty0 - RAD + tok / HW, xx = tx0 - RAD + tok % HW;
            uint4 val = make_uint4(0u, 0u, 0u, 0u);
            if (piece * VEC < p.d_valid && yy >= 0 && yy < p.grid_h && xx >= 0 && xx < p.grid_w)
                val = *reinterpret_cast<const uint4*>(
                    v + in_off + (static_cast<long long>(yy) * p.grid_w + xx) * p.in.n + piece * VEC);
            *reinterpret_cast<uint4*>(vh + static_cast<size_t>(tok) * D + piece * VEC) = val;
        }
        for (int idx = tid; idx < kApplyTokens * LPR; idx += 256) {
            const int tok = idx / LPR, piece = idx % LPR;
            const int yy = ty0 + tok / kApplyTW, xx = tx0 + tok % kApplyTW;
            uint4 val = make_uint4(0u, 0u, 0u, 0u);
            if (piece * VEC < p.d_valid && yy < p.grid_h && xx < p.grid_w)
                val = *reinterpret_cast<const uint4*>(
                    g + out_off + (static_cast<long long>(yy) * p.grid_w + xx) * p.out.n + piece * VEC);
            *reinterpret_cast<uint4*>(gt + static_cast<size_t>(tok) * D + piece * VEC) = val;
        }
        __syncthreads();
#pragma unroll 2
        for (int tok = 0; tok < kApplyTokens; ++tok) {
            // all LDS reads of a token first, then the arithmetic: the reads overlap each other
            const Pair gp = *reinterpret_cast<const Pair*>(gt + tok * D + c);
            const T* base = vh + ((tok / kApplyTW) * HW + tok % kApplyTW) * D + c;
            Pair vp[TAPS];
#pragma unroll
            for (int i = 0; i < TAPS; ++i) vp[i] = *reinterpret_cast<const Pair*>(base + tap_off[i]);
            __builtin_amdgcn_sched_barrier(0);
            const float g0 = IO<T>::to_f32(gp.a), g1 = IO<T>::to_f32(gp.b);
            gsum[0] += g0;
            gsum[1] += g1;
#pragma unroll
            for (int i = 0; i < TAPS; ++i) {
                acc[i][0] = fmaf(g0, IO<T>::to_f32(vp[i].a), acc[i][0]);
                acc[i][1] = fmaf(g1, IO<T>::to_f32(vp[i].b), acc[i][1]);
            }
        }
    }
    float* o = part_out + (static_cast<size_t>(unit) * p.chunks + blockIdx.x) * NT * D;
#pragma unroll
    for (int i = 0; i < TAPS; ++i) {
        const int e = part + TPC * i;
        if (e < KS * KS) {
            o[e * D + c] = acc[i][0];
            o[e * D + c + 1] = acc[i][1];
        }
    }
    if (part == 0) {
        o[KS * KS * D + c] = gsum[0];
        o[KS * KS * D + c + 1] = gsum[1];
    }
}

// grid = (ceil(heads * d * (taps + 1) / 256)), block = 256: sums the partial filter gradients
// over the batch and the chunks, in order, into dw [heads][d][taps] and dbias [heads][d] (may
// be null).  part: [B * heads][chunks][taps + 1][D].
__global__ __launch_bounds__(256) void bwd_filter_combine_kernel(const float* __restrict__ part,
                                                                 float* __restrict__ dw,
                                                                 float* __restrict__ dbias, int B,
                                                                 int heads, int d, int D, int taps,
                                                                 int chunks)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int nt = taps + 1;
    if (i >= heads * d * nt) return;
    const int ch = i % d, e = (i / d) % nt, h = i / (nt * d);  // neighbours read neighbours
    float s = 0.f;
    for (int b = 0; b < B; ++b) {
        const float* src = part + (static_cast<size_t>(b) * heads + h) * chunks * nt * D + e * D + ch;
        s += sum_partials(src, chunks, static_cast<size_t>(nt) * D);
    }
    if (e < taps) dw[(static_cast<size_t>(h) * d + ch) * taps + e] = s;
    else if (dbias) dbias[h * d + ch] = s;
}

}  // namespace castling
