// Backward pass of the layer: the gradients of Eq. 3 / 8 / 9 with respect to q, k, v, the DWConv
// filters and their bias, given g = dLoss/dout.
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
// per-row kernel (a, b, dq; dk) in a vector-ALU form (any I/O type and head width, fp32 products)
// and a matrix-core form (16-bit, 32 or 64 channels), the filter gradient and small helpers.
#pragma once

#include "apply_generic.hpp"
#include "common.hpp"
#include "formats.hpp"

namespace castling {

struct BwdRowsParams {
    int N;           // tokens per unit of k and v (the sums of Eq. 3 run over them)
    int rows;        // rows this launch walks: N, or the number of pooled queries
    int tiles;       // ceil(rows / 64)
    int norm_none;
    int residual_q;  // QUERY: dq gains g
    int d_valid;     // features per head in memory (<= D)
    float eps;
    // a is stored times ascale (N with the normaliser: a_t = g_t / den_t is of the order g / N,
    // below the normal range of fp16 for long sequences; 1 without), so the state of (q, a) is
    // ascale times S', va'.  mscale: factor on the state matrix as it is loaded (1/pi for the
    // forward state, 1/(pi ascale) for the state of (q, a)).
    float ascale, mscale;
    TensorStrides in, out;  // of k, v, a and the gradient of k; of g
    TensorStrides xs;       // of x and dx: those of q (QUERY) or `in`
    // Downsampling layers (QUERY, up_s = 2): query row t = (yq, xq) of the up_wq-wide coarse grid
    // stands at token (up_s yq) up_w + up_s xq of the fine grid; a is written to that row of
    // its buffer and q, g are copied to the same row of q_up, g_up (all three with the layout
    // `in`, zero elsewhere), so that the later passes run on the fine grid as they are.
    int up_s, up_wq, up_w;
    void* q_up;
    void* g_up;
};

// row of the a buffer for query row n (see BwdRowsParams::up_s)
__device__ __forceinline__ int bwd_a_row(const BwdRowsParams& p, int n)
{
    return p.up_s ? (n / p.up_wq) * p.up_s * p.up_w + (n % p.up_wq) * p.up_s : n;
}

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
    const long long x_off = unit_offset(unit, heads, p.xs);

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
        if (n < p.rows && lcol < p.d_valid) {
            const uint4 raw = *reinterpret_cast<const uint4*>(x + x_off + n * p.xs.n + lcol);
            IO<T>::widen16(raw, xv);
            if (!QUERY) IO<T>::load16(y + in_off + n * p.in.n + lcol, yv);
            if (QUERY && p.up_s)  // the query row on its place in the fine grid
                *reinterpret_cast<uint4*>(static_cast<T*>(p.q_up) + in_off +
                                          bwd_a_row(p, n) * p.in.n + lcol) = raw;
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
            const bool live = n < p.rows && tj * RJ < p.d_valid;
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
            if (live) {
                const long long at = in_off + bwd_a_row(p, n) * p.in.n + tj * RJ;
                store_piece<T, RJ>(a_out + at, av);
                if (p.up_s) store_piece<T, RJ>(static_cast<T*>(p.g_up) + at, gown[t]);
            }
            if (tj == 0) bs[tt * 4 + t] = n < p.rows ? bt : 0.f;
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
        if (n < p.rows && tj * RJ < p.d_valid) {
            float r[RJ];
#pragma unroll
            for (int j = 0; j < RJ; ++j) {
                r[j] = (dxh[t][j] - xh[j] * dot) * inv[tl];
                if (QUERY && p.residual_q) r[j] += gown[t][j];
            }
            store_piece<T, RJ>(dx + x_off + n * p.xs.n + tj * RJ, r);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The per-row kernel on the matrix cores (16-bit I/O, D = 32 or 64): the two D x D products of a
// tile of 64 rows run as 16x16x32 MFMAs, wave w on rows 16 w .. 16 w + 15.  Operands: rows as
// stored (exact) and the state matrix times table_scale rounded once to the I/O format, as in
// the forward's pass 2 -- here followed by a second 16-bit term holding what the rounding cut off
// (M = M_hi + M_lo, a = a_hi + a_lo; the lo x lo products are dropped), since a gradient has no
// exactly accumulated part to hide the operand rounding behind.  The block
// loads the state once and walks `tiles_per_block` tiles; every row buffer in LDS is private
// to one wave.  kb_part holds one share per wave: [unit][4 tiles][D].
// MFMA layouts (lane l): A[m][k]: m = l % 16, k = 8 (l / 16) + 0..7;  B[k][n]: n = l % 16, same k;
// C[m][n]: n = l % 16, m = 4 (l / 16) + r, r = 0..3.
// Orders the LDS accesses of one wave for the compiler where a buffer is written through one type
// and read through another (the hardware runs a wave's LDS instructions in order).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_wave_barrier();
    asm volatile("" ::: "memory");
}

template <int D>
constexpr size_t bwd_rows_mfma_lds_bytes()
{
    return 2 * (4 * static_cast<size_t>(D) * (D + 8) + 4 * kBwdTokens * (D + 8)) +
           sizeof(float) * (2 * D + 4 * 4 * 16);
}

template <typename X, int D, bool QUERY>
__global__ __launch_bounds__(256) void bwd_rows_mfma_kernel(const uint16_t* __restrict__ x,
                                                            const uint16_t* __restrict__ y,
                                                            const float* __restrict__ state,
                                                            const float* __restrict__ vec,
                                                            uint16_t* __restrict__ a_out,
                                                            float* __restrict__ kb_part,
                                                            uint16_t* __restrict__ dx, int heads,
                                                            BwdRowsParams p, int tiles_per_block)
{
    constexpr int P = D + 8;  // row pitch of the LDS tiles, 16-bit elements
    constexpr int NT = D / 16, KSTEPS = D / 32;
    constexpr int PIECES = D / 8;        // 16-byte pieces per row
    constexpr int RP = 64 / PIECES;      // rows one pass of a wave loads
    constexpr int PASSES = 16 / RP;
    using L = StateLayout<D>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint16_t* Ms = reinterpret_cast<uint16_t*>(lds_raw);  // [D][P]  M[i][c], rounded
    uint16_t* Mt = Ms + D * P;                            // [D][P]  M[i][c] at [c][i]
    uint16_t* Msl = Mt + D * P;                           // the same two for M minus its rounding
    uint16_t* Mtl = Msl + D * P;
    uint16_t* xr = Mtl + D * P;                           // [64][P] rows of x as stored
    uint16_t* ar = xr + kBwdTokens * P;                   // [64][P] rows of a (times ascale) / of v
    uint16_t* al = ar + kBwdTokens * P;                   // [64][P] a minus its rounding (QUERY)
    uint16_t* gr = al + kBwdTokens * P;                   // [64][P] rows of g; then the result rows
    float* vk = reinterpret_cast<float*>(gr + kBwdTokens * P);  // ksum / pi  (kb' / pi)
    float* vs = vk + D;                                          // vsum / 2
    float* rowf = vs + D;                                        // [wave][inv, den, small, b][16]

    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int unit = blockIdx.y;
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long out_off = unit_offset(unit, heads, p.out);
    const long long x_off = unit_offset(unit, heads, p.xs);
    const float ts = X::table_scale(p.N), us = X::table_unscale(p.N);
    const float post = us / p.ascale;

    const float* gs = state + static_cast<size_t>(unit) * L::SIZE;
    block_stage<D * D, float>(
        tid, [&](int i) { return gs[L::S + i]; },
        [&](int i, float s) {
            const uint16_t m = static_cast<uint16_t>(X::pack(s * ts, 0.f));
            const uint16_t ml = static_cast<uint16_t>(X::pack(s * ts - X::one(m), 0.f));
            Ms[(i / D) * P + i % D] = m;
            Mt[(i % D) * P + i / D] = m;
            Msl[(i / D) * P + i % D] = ml;
            Mtl[(i % D) * P + i / D] = ml;
        });
    if (tid < D) {
        vk[tid] = (QUERY ? gs[L::KSUM + tid] : vec[static_cast<size_t>(unit) * D + tid]) * kInvPi;
        vs[tid] = 0.5f * gs[L::VSUM + tid];
    }
    __syncthreads();

    float* w_inv = rowf + wave * 64;
    float* w_den = w_inv + 16;
    float* w_small = w_den + 16;
    float* w_b = w_small + 16;
    const int cl = lane % 16, g4 = lane / 16;       // MFMA layouts
    const int lrow = lane / PIECES, piece = lane % PIECES;  // row I/O
    uint16_t* my_x = xr + wave * 16 * P;
    uint16_t* my_a = ar + wave * 16 * P;
    uint16_t* my_al = al + wave * 16 * P;
    uint16_t* my_g = gr + wave * 16 * P;

    // the rows of a tile are loaded one tile ahead: their latency passes behind the previous
    // tile's work
    u32x4_t xnext[PASSES], ynext[PASSES];
    auto fetch_rows = [&](int tile) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int n = tile * kBwdTokens + wave * 16 + ps * RP + lrow;
            xnext[ps] = u32x4_t{0u, 0u, 0u, 0u};
            ynext[ps] = u32x4_t{0u, 0u, 0u, 0u};
            if (tile < p.tiles && n < p.rows) {
                xnext[ps] = *reinterpret_cast<const u32x4_t*>(x + x_off + n * p.xs.n + piece * 8);
                ynext[ps] = QUERY ? *reinterpret_cast<const u32x4_t*>(y + out_off + n * p.out.n + piece * 8)
                                  : *reinterpret_cast<const u32x4_t*>(y + in_off + n * p.in.n + piece * 8);
            }
        }
    };
    fetch_rows(blockIdx.x * tiles_per_block);

    for (int it = 0; it < tiles_per_block; ++it) {
        const int tile = blockIdx.x * tiles_per_block + it;
        if (tile >= p.tiles) break;
        const int n0 = tile * kBwdTokens + wave * 16;

        // ---- rows in: x -> xr, g -> gr (QUERY) or v -> ar; norms, den
        u32x4_t xkeep[PASSES];
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int row = ps * RP + lrow;
            const u32x4_t xv = xnext[ps], yv = ynext[ps];
            xkeep[ps] = xv;
            if (QUERY && p.up_s && n0 + row < p.rows) {  // q and g on their place in the fine grid
                const long long at = in_off + bwd_a_row(p, n0 + row) * p.in.n + piece * 8;
                *reinterpret_cast<u32x4_t*>(static_cast<uint16_t*>(p.q_up) + at) = xv;
                *reinterpret_cast<u32x4_t*>(static_cast<uint16_t*>(p.g_up) + at) = yv;
            }
            *reinterpret_cast<u32x4_t*>(my_x + row * P + piece * 8) = xv;
            *reinterpret_cast<u32x4_t*>((QUERY ? my_g : my_a) + row * P + piece * 8) = yv;
            float ss = 0.f, qk = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = X::lo(xv[e]), hi = X::hi(xv[e]);
                ss = fmaf(lo, lo, fmaf(hi, hi, ss));
                qk = fmaf(lo, vk[piece * 8 + 2 * e], fmaf(hi, vk[piece * 8 + 2 * e + 1], qk));
            }
            ss = row_group_sum<PIECES>(ss);
            qk = row_group_sum<PIECES>(qk);
            const float nrm = sqrtf(ss);
            const float r = 1.0f / fmaxf(nrm, p.eps);
            if (piece == 0) {
                w_inv[row] = r;
                w_den[row] = 0.5f * static_cast<float>(p.N) + r * qk;
                w_small[row] = nrm < p.eps ? 1.f : 0.f;
                w_b[row] = 1.f;
            }
        }
        if (it + 1 < tiles_per_block) fetch_rows(tile + 1);
        wave_lds_fence();
        float inv_r[4], b_r[4], small_r[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            inv_r[r] = w_inv[4 * g4 + r];
            small_r[r] = w_small[4 * g4 + r];
            b_r[r] = 1.f;
        }

        float gC[NT][4];  // QUERY: g in the C layout (kept for the residual)
        if (QUERY) {
            // ---- num = vs + inv us (q M): product 1, B = columns of M read from Mt
            f32x4_t acc1[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc1[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const u32x4_t A = *reinterpret_cast<const u32x4_t*>(my_x + cl * P + ks * 32 + 8 * g4);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int off = (nt * 16 + cl) * P + ks * 32 + 8 * g4;
                    acc1[nt] = X::mfma16(A, *reinterpret_cast<const u32x4_t*>(Mt + off), acc1[nt]);
                    acc1[nt] = X::mfma16(A, *reinterpret_cast<const u32x4_t*>(Mtl + off), acc1[nt]);
                }
            }
            float rden[4], gl[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) rden[r] = 1.0f / w_den[4 * g4 + r];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int c = nt * 16 + cl;
                    gC[nt][r] = X::one(my_g[(4 * g4 + r) * P + c]);
                    const float lin = (vs[c] + inv_r[r] * us * acc1[nt][r]) * rden[r];
                    gl[r] = fmaf(gC[nt][r], lin, gl[r]);
                }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                gl[r] = row_group_sum<16>(gl[r]);  // g_t . lin_t over all features
                b_r[r] = p.norm_none ? 0.f : -gl[r] * rden[r];
                if (cl == 0) w_b[4 * g4 + r] = b_r[r];
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float a0 = (p.norm_none ? gC[nt][r] : gC[nt][r] * rden[r]) * p.ascale;
                    const uint16_t ah = static_cast<uint16_t>(X::pack(a0, 0.f));
                    my_a[(4 * g4 + r) * P + nt * 16 + cl] = ah;
                    my_al[(4 * g4 + r) * P + nt * 16 + cl] =
                        static_cast<uint16_t>(X::pack(a0 - X::one(ah), 0.f));
                }
            wave_lds_fence();
            // ---- rows of a out; this wave's share of kb' = sum_t q_hat_t b_t
            float kbp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int row = ps * RP + lrow, n = n0 + row;
                if (n < p.rows)
                    *reinterpret_cast<u32x4_t*>(a_out + in_off + bwd_a_row(p, n) * p.in.n + piece * 8) =
                        *reinterpret_cast<const u32x4_t*>(my_a + row * P + piece * 8);
                const float wgt = w_inv[row] * w_b[row];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    kbp[2 * e] = fmaf(X::lo(xkeep[ps][e]), wgt, kbp[2 * e]);
                    kbp[2 * e + 1] = fmaf(X::hi(xkeep[ps][e]), wgt, kbp[2 * e + 1]);
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int m = PIECES; m < 64; m <<= 1) kbp[e] += __shfl_xor(kbp[e], m, 64);
            if (lrow == 0) {
                float* o = kb_part + ((static_cast<size_t>(unit) * p.tiles + tile) * 4 + wave) * D + piece * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = kbp[e];
            }
        }

        // ---- dx_hat = post (a M^T) + vk b: product 2, B = rows of M
        f32x4_t acc2[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc2[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4_t A = *reinterpret_cast<const u32x4_t*>(my_a + cl * P + ks * 32 + 8 * g4);
            u32x4_t Al = {0u, 0u, 0u, 0u};
            if (QUERY) Al = *reinterpret_cast<const u32x4_t*>(my_al + cl * P + ks * 32 + 8 * g4);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int off = (nt * 16 + cl) * P + ks * 32 + 8 * g4;
                const u32x4_t B = *reinterpret_cast<const u32x4_t*>(Ms + off);
                acc2[nt] = X::mfma16(A, B, acc2[nt]);
                acc2[nt] = X::mfma16(A, *reinterpret_cast<const u32x4_t*>(Msl + off), acc2[nt]);
                if (QUERY) acc2[nt] = X::mfma16(Al, B, acc2[nt]);  // (rows of v are exact as stored)
            }
        }
        float dxh[NT][4], xh[NT][4], dot[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = nt * 16 + cl;
                dxh[nt][r] = fmaf(acc2[nt][r], post, vk[i] * b_r[r]);
                xh[nt][r] = X::one(my_x[(4 * g4 + r) * P + i]) * inv_r[r];
                dot[r] = fmaf(xh[nt][r], dxh[nt][r], dot[r]);
            }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dot[r] = row_group_sum<16>(dot[r]);
            if (small_r[r] != 0.f) dot[r] = 0.f;  // below the floor the row is x / eps: no projection
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float res = (dxh[nt][r] - xh[nt][r] * dot[r]) * inv_r[r];
                if (QUERY && p.residual_q) res += gC[nt][r];
                my_g[(4 * g4 + r) * P + nt * 16 + cl] = static_cast<uint16_t>(X::pack(res, 0.f));
            }
        wave_lds_fence();
        // ---- result rows out
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int row = ps * RP + lrow, n = n0 + row;
            if (n < p.rows)
                *reinterpret_cast<u32x4_t*>(dx + x_off + n * p.xs.n + piece * 8) =
                    *reinterpret_cast<const u32x4_t*>(my_g + row * P + piece * 8);
        }
        wave_lds_fence();
    }
}

// grid = (units), block = 1024: kb[unit][i] = sum over the shares kb_part[unit][share][i].  The
// 1024 / D slices of the block each sum a contiguous run of shares in order; slice 0 adds the
// slice sums in order (a fixed order of additions: the result is deterministic).
__global__ __launch_bounds__(1024) void bwd_vec_combine_kernel(const float* __restrict__ kb_part,
                                                               float* __restrict__ kb, int parts, int D)
{
    __shared__ float red[1024];
    const int tid = threadIdx.x;
    const int i = tid % D, sl = tid / D, nsl = 1024 / D;
    const int per = (parts + nsl - 1) / nsl;
    const int p0 = sl * per;
    const int cnt = parts - p0 < per ? parts - p0 : per;
    const float* src = kb_part + (static_cast<size_t>(blockIdx.x) * parts + p0) * D + i;
    red[tid] = cnt > 0 ? sum_partials(src, cnt, D) : 0.f;
    __syncthreads();
    if (sl == 0) {
        float s = red[i];
        for (int k = 1; k < nsl; ++k) s += red[k * D + i];
        kb[static_cast<size_t>(blockIdx.x) * D + i] = s;
    }
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

// grid = (ceil(rows * d / VEC / 256), units), block = 256: row t = (yq, xq) of a wq-wide coarse grid
// of `src` to token (2 yq) w + 2 xq of `dst` (16-byte pieces).
template <typename T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                           int rows, int d, int heads, TensorStrides ss,
                                                           TensorStrides ds, int wq, int w)
{
    constexpr int VEC = IO<T>::VEC;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int per_row = d / VEC;
    if (i >= rows * per_row) return;
    const int t = i / per_row, piece = i % per_row;
    const long long to = (t / wq) * 2ll * w + (t % wq) * 2;
    *reinterpret_cast<uint4*>(dst + unit_offset(blockIdx.y, heads, ds) + to * ds.n + piece * VEC) =
        *reinterpret_cast<const uint4*>(src + unit_offset(blockIdx.y, heads, ss) + t * ss.n + piece * VEC);
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

template <typename T>
struct alignas(2 * sizeof(T)) ChannelPair {
    T a, b;
};

constexpr int kBwdFilterThreads = 512;

// 16-byte piece idx of a tile's LDS image: the halo tile of v ([HH][HW][D], zero outside the
// grid) and behind it the 4 x 16 tile of g.
template <typename T, int D, int KS>
__device__ __forceinline__ uint4 bwd_filter_piece(const T* __restrict__ v, const T* __restrict__ g,
                                                  const BwdFilterParams& p, long long in_off,
                                                  long long out_off, int tile, int idx)
{
    constexpr int VEC = IO<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int HH = kApplyTH + KS - 1, HW = kApplyTW + KS - 1;
    const int ty0 = (tile / p.tiles_x) * kApplyTH, tx0 = (tile % p.tiles_x) * kApplyTW;
    const int tok = idx / LPR, piece = idx % LPR;
    const bool halo = tok < HH * HW;
    const int gtok = tok - HH * HW;
    const int yy = halo ? ty0 - KS / 2 + tok / HW : ty0 + gtok / kApplyTW;
    const int xx = halo ? tx0 - KS / 2 + tok % HW : tx0 + gtok % kApplyTW;
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if (idx < (HH * HW + kApplyTokens) * LPR && piece * VEC < p.d_valid && yy >= 0 && yy < p.grid_h &&
        xx >= 0 && xx < p.grid_w) {
        const long long at = (static_cast<long long>(yy) * p.grid_w + xx);
        val = halo ? *reinterpret_cast<const uint4*>(v + in_off + at * p.in.n + piece * VEC)
                   : *reinterpret_cast<const uint4*>(g + out_off + at * p.out.n + piece * VEC);
    }
    return val;
}

// Two LDS images (the next tile's loads are in flight while this one is worked on) where a
// thread holds few pieces of an image and both fit.
template <typename T, int D, int KS>
constexpr bool bwd_filter_double_buffered()
{
    const size_t image = sizeof(T) * ((kApplyTH + KS - 1) * (kApplyTW + KS - 1) + kApplyTokens) * D;
    return image / 16 <= 6 * kBwdFilterThreads && 2 * image <= 100 * 1024;
}

template <typename T, int D, int KS>
constexpr size_t bwd_filter_lds_bytes()
{
    // halo tile of v and tile of g; afterwards the block's sums [KS * KS + 1][D] in fp32
    const size_t tiles = sizeof(T) * ((kApplyTH + KS - 1) * (kApplyTW + KS - 1) + kApplyTokens) * D *
                         (bwd_filter_double_buffered<T, D, KS>() ? 2 : 1);
    const size_t sums = sizeof(float) * (KS * KS + 1) * D;
    return tiles > sums ? tiles : sums;
}

// Filter and bias gradients: dw[c][dy][dx] = sum over tokens of g[t][c] v[t + (dy, dx) - r][c],
// dbias[c] = sum of g[t][c].  grid = (chunks, units), block = 512, dynamic LDS =
// bwd_filter_lds_bytes; v, g point at the first grid token.  The block walks its 4 x 16 tiles
// (halo tile of v and tile of g in LDS).  A thread owns two channels, one tile row ty and the
// filter rows dy = part / 4, part / 4 + TPC / 4, ... (part = tid / (D / 2), TPC = 1024 / D parts):
// per tile and half row it reads 8 tokens of g's row ty and, per filter row, the KS + 7 tokens
// of v's row ty + dy they meet, and slides the one over the other in registers.  At the end the four tile
// rows meet in LDS in the order ty = 0, 1, 2, 3 (a fixed order of additions) and the block writes
// part_out[unit][chunk][tap][D] (tap KS * KS: the sum of g, the bias gradient).
template <typename T, int D, int KS>
__global__ __launch_bounds__(kBwdFilterThreads) void bwd_filter_kernel(const T* __restrict__ v,
                                                                       const T* __restrict__ g,
                                                                       float* __restrict__ part_out,
                                                                       int heads, BwdFilterParams p)
{
    constexpr int NTHR = kBwdFilterThreads;
    constexpr int VEC = IO<T>::VEC;
    constexpr int HH = kApplyTH + KS - 1, HW = kApplyTW + KS - 1;
    using Pair = ChannelPair<T>;
    constexpr int TPC = 2 * NTHR / D;              // threads per pair of channels
    constexpr int DYS = TPC / 4;                   // filter rows taken at a time
    constexpr int IPT = (KS + DYS - 1) / DYS;      // filter rows per thread
    constexpr int NT = KS * KS + 1;                // taps and the bias
    static_assert(TPC % 4 == 0, "a thread keeps one tile row");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    T* vh = reinterpret_cast<T*>(lds_raw);  // image(s): [HH][HW][D] of v, then [4 x 16][D] of g

    const int tid = threadIdx.x;
    const int unit = blockIdx.y;
    const int c = 2 * (tid % (D / 2)), part = tid / (D / 2);
    const int ty = part % 4, dy0 = part / 4;
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long out_off = unit_offset(unit, heads, p.out);

    float acc[IPT][KS][2], gsum[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < IPT; ++i)
#pragma unroll
        for (int dx = 0; dx < KS; ++dx) acc[i][dx][0] = acc[i][dx][1] = 0.f;

    constexpr bool DB = bwd_filter_double_buffered<T, D, KS>();
    constexpr int IMAGE = (HH * HW + kApplyTokens) * D;     // elements of one LDS image
    constexpr int PIECES = (IMAGE / VEC + NTHR - 1) / NTHR;  // 16-byte pieces per thread
    uint4 pre[DB ? PIECES : 1];
    int buf = 0;
    if constexpr (DB) {
        if (static_cast<int>(blockIdx.x) < p.n_tiles) {
#pragma unroll
            for (int k = 0; k < PIECES; ++k)
                pre[k] = bwd_filter_piece<T, D, KS>(v, g, p, in_off, out_off, blockIdx.x, tid + NTHR * k);
#pragma unroll
            for (int k = 0; k < PIECES; ++k)
                if (tid + NTHR * k < IMAGE / VEC)
                    *reinterpret_cast<uint4*>(vh + static_cast<size_t>(tid + NTHR * k) * VEC) = pre[k];
        }
        __syncthreads();
    }
    for (int tile = blockIdx.x; tile < p.n_tiles; tile += p.chunks) {
        if constexpr (DB) {
            // the next tile's loads go out now and land in the other image after this tile's work
            if (tile + p.chunks < p.n_tiles) {
#pragma unroll
                for (int k = 0; k < PIECES; ++k)
                    pre[k] = bwd_filter_piece<T, D, KS>(v, g, p, in_off, out_off, tile + p.chunks,
                                                        tid + NTHR * k);
            }
        } else {
            __syncthreads();  // the previous tile's reads are done
            block_stage<IMAGE / VEC, uint4, NTHR, 6>(
                tid,
                [&](int idx) { return bwd_filter_piece<T, D, KS>(v, g, p, in_off, out_off, tile, idx); },
                [&](int idx, uint4 val) {
                    *reinterpret_cast<uint4*>(vh + static_cast<size_t>(idx) * VEC) = val;
                });
            __syncthreads();
        }
        const T* vcur = vh + buf * IMAGE;
        const T* gcur = vcur + HH * HW * D;

        // half a tile row at a time (fewer registers): 8 tokens of g against KS + 7 tokens of v
#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            constexpr int TXH = kApplyTW / 2, WINH = TXH + KS - 1;
            float g0[TXH], g1[TXH];
#pragma unroll
            for (int tx = 0; tx < TXH; ++tx) {
                const Pair gp = *reinterpret_cast<const Pair*>(gcur + (ty * kApplyTW + half * TXH + tx) * D + c);
                g0[tx] = IO<T>::to_f32(gp.a);
                g1[tx] = IO<T>::to_f32(gp.b);
            }
            if (dy0 == 0) {
#pragma unroll
                for (int tx = 0; tx < TXH; ++tx) {
                    gsum[0] += g0[tx];
                    gsum[1] += g1[tx];
                }
            }
#pragma unroll
            for (int i = 0; i < IPT; ++i) {
                const int dy = dy0 + DYS * i;
                if (dy < KS) {  // (the same for all lanes of a wave where D >= 32)
                    float w0[WINH], w1[WINH];
#pragma unroll
                    for (int x = 0; x < WINH; ++x) {
                        const Pair wp = *reinterpret_cast<const Pair*>(
                            vcur + ((ty + dy) * HW + half * TXH + x) * D + c);
                        w0[x] = IO<T>::to_f32(wp.a);
                        w1[x] = IO<T>::to_f32(wp.b);
                    }
#pragma unroll
                    for (int tx = 0; tx < TXH; ++tx)
#pragma unroll
                        for (int dx = 0; dx < KS; ++dx) {
                            acc[i][dx][0] = fmaf(g0[tx], w0[tx + dx], acc[i][dx][0]);
                            acc[i][dx][1] = fmaf(g1[tx], w1[tx + dx], acc[i][dx][1]);
                        }
                }
                __builtin_amdgcn_sched_barrier(0);  // one window in registers at a time
            }
        }
        if constexpr (DB) {
            if (tile + p.chunks < p.n_tiles) {
                T* vnext = vh + (buf ^ 1) * IMAGE;
#pragma unroll
                for (int k = 0; k < PIECES; ++k)
                    if (tid + NTHR * k < IMAGE / VEC)
                        *reinterpret_cast<uint4*>(vnext + static_cast<size_t>(tid + NTHR * k) * VEC) = pre[k];
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    // the four tile rows of a tap meet in LDS, in order
    __syncthreads();
    float* sums = reinterpret_cast<float*>(lds_raw);  // [NT][D]
#pragma unroll 1
    for (int ph = 0; ph < 4; ++ph) {
        if (ty == ph) {
#pragma unroll
            for (int i = 0; i < IPT; ++i) {
                const int dy = dy0 + DYS * i;
                if (dy < KS) {
#pragma unroll
                    for (int dx = 0; dx < KS; ++dx) {
                        float* s = sums + (dy * KS + dx) * D + c;
                        s[0] = ph == 0 ? acc[i][dx][0] : s[0] + acc[i][dx][0];
                        s[1] = ph == 0 ? acc[i][dx][1] : s[1] + acc[i][dx][1];
                    }
                }
            }
            if (dy0 == 0) {
                float* s = sums + KS * KS * D + c;
                s[0] = ph == 0 ? gsum[0] : s[0] + gsum[0];
                s[1] = ph == 0 ? gsum[1] : s[1] + gsum[1];
            }
        }
        __syncthreads();
    }
    float* o = part_out + (static_cast<size_t>(unit) * p.chunks + blockIdx.x) * NT * D;
    for (int idx = tid; idx < NT * D; idx += NTHR) o[idx] = sums[idx];
}

// ---------------------------------------------------------------------------------------------
// The filter gradient for 16-bit I/O on two-element dot products (v_dot2c_f32_bf16 / _f16): the
// sum over tokens runs over pairs of neighbouring tokens of one channel, so LDS holds the tiles
// channel-major (tokens of a channel contiguous, two per 32-bit word; the channel stride is an odd
// number of words: lanes = channels read conflict-free) -- the staging transposes the 16-byte
// pieces of 8 channels into eight 2-byte writes.  A thread owns one channel, one tile row ty
// and the filter rows dy = part / 4, part / 4 + TPC / 4, ... (part = tid / D, TPC = 512 / D); per
// tile it reads the 8 words of g's row ty and, per filter row, the words of v's row ty + dy, forms
// the odd-aligned pairs with one funnel shift each, and does 8 dot products per tap (half the
// FMAs of the fp32 form and no conversions).  Same partial layout, same fixed order of additions
// as bwd_filter_kernel.
template <int D, int KS>
struct FilterDot2Layout {
    static constexpr int HH = kApplyTH + KS - 1, HW = kApplyTW + KS - 1;
    static constexpr int ROW = HW / 2;                 // words per halo row of one channel
    static constexpr int CS = (HH * ROW) | 1;          // words per channel of v (odd)
    static constexpr int GS = (kApplyTokens / 2) | 1;  // words per channel of g (odd)
    static constexpr int IMAGE = D * (CS + GS);        // words of one image
    static constexpr int ITEMS = (HH * HW + kApplyTokens) * (D / 8);  // 16-byte pieces of one image
    static constexpr int PIECES = (ITEMS + kBwdFilterThreads - 1) / kBwdFilterThreads;
    static constexpr bool DB = PIECES <= 6 && 2 * IMAGE * 4 <= 110 * 1024;
    static_assert(HW % 2 == 0, "rows hold whole pairs of tokens");
};

template <int D, int KS>
constexpr size_t bwd_filter_dot2_lds_bytes()
{
    using L = FilterDot2Layout<D, KS>;
    const size_t tiles = static_cast<size_t>(L::IMAGE) * 4 * (L::DB ? 2 : 1);
    const size_t sums = sizeof(float) * (KS * KS + 1) * D;
    return tiles > sums ? tiles : sums;
}

template <typename X, int D, int KS>
__global__ __launch_bounds__(kBwdFilterThreads) void bwd_filter_dot2_kernel(
    const uint16_t* __restrict__ v, const uint16_t* __restrict__ g, float* __restrict__ part_out,
    int heads, BwdFilterParams p)
{
    using L = FilterDot2Layout<D, KS>;
    constexpr int NTHR = kBwdFilterThreads;
    constexpr int HH = L::HH, HW = L::HW, ROW = L::ROW, CS = L::CS, GS = L::GS;
    constexpr int TPC = NTHR / D;                  // threads per channel
    constexpr int DYS = TPC / 4;                   // filter rows taken at a time
    constexpr int IPT = (KS + DYS - 1) / DYS;      // filter rows per thread
    constexpr int NT = KS * KS + 1;                // taps and the bias
    constexpr bool DB = L::DB;
    constexpr int PIECES = L::PIECES;
    static_assert(TPC % 4 == 0, "a thread keeps one tile row");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint32_t* img = reinterpret_cast<uint32_t*>(lds_raw);

    const int tid = threadIdx.x;
    const int unit = blockIdx.y;
    const int c = tid % D, part = tid / D;
    const int ty = part % 4, dy0 = part / 4;
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long out_off = unit_offset(unit, heads, p.out);
    const uint32_t ones = opaque_u32(X::kOneLo | X::kOneHi);  // (kept out of the inline constants)

    float acc[IPT][KS], gsum = 0.f;
#pragma unroll
    for (int i = 0; i < IPT; ++i)
#pragma unroll
        for (int dx = 0; dx < KS; ++dx) acc[i][dx] = 0.f;

    // piece idx of a tile's image from global memory / into the channel-major LDS image
    auto load_piece16 = [&](int tile, int idx) {
        return bwd_filter_piece<uint16_t, D, KS>(v, g, p, in_off, out_off, tile, idx);
    };
    auto store_piece16 = [&](uint32_t* dst_img, int idx, uint4 val) {
        if (idx >= L::ITEMS) return;
        const int tok = idx / (D / 8), piece = idx % (D / 8);
        const bool halo = tok < HH * HW;
        const int t2 = halo ? tok : tok - HH * HW;
        uint16_t* base = reinterpret_cast<uint16_t*>(dst_img + (halo ? 0 : D * CS)) + t2;
        const int cs2 = 2 * (halo ? CS : GS);  // channel stride in 16-bit elements
        const uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            base[(piece * 8 + 2 * e) * cs2] = static_cast<uint16_t>(w[e]);
            base[(piece * 8 + 2 * e + 1) * cs2] = static_cast<uint16_t>(w[e] >> 16);
        }
    };

    uint4 pre[DB ? PIECES : 1];
    int buf = 0;
    if constexpr (DB) {
        if (static_cast<int>(blockIdx.x) < p.n_tiles) {
#pragma unroll
            for (int k = 0; k < PIECES; ++k) pre[k] = load_piece16(blockIdx.x, tid + NTHR * k);
#pragma unroll
            for (int k = 0; k < PIECES; ++k) store_piece16(img, tid + NTHR * k, pre[k]);
        }
        __syncthreads();
    }
    for (int tile = blockIdx.x; tile < p.n_tiles; tile += p.chunks) {
        if constexpr (DB) {
            // the next tile's loads go out now and land in the other image after this tile's work
            if (tile + p.chunks < p.n_tiles) {
#pragma unroll
                for (int k = 0; k < PIECES; ++k) pre[k] = load_piece16(tile + p.chunks, tid + NTHR * k);
            }
        } else {
            __syncthreads();  // the previous tile's reads are done
            block_stage<L::ITEMS, uint4, NTHR, 6>(
                tid, [&](int idx) { return load_piece16(tile, idx); },
                [&](int idx, uint4 val) { store_piece16(img, idx, val); });
            __syncthreads();
        }
        const uint32_t* vcur = img + buf * L::IMAGE + c * CS;
        const uint32_t* gcur = img + buf * L::IMAGE + D * CS + c * GS + ty * (kApplyTW / 2);

        uint32_t G[kApplyTW / 2];  // pairs of tokens of g's row ty
#pragma unroll
        for (int j = 0; j < kApplyTW / 2; ++j) G[j] = gcur[j];
        if (dy0 == 0) {
#pragma unroll
            for (int j = 0; j < kApplyTW / 2; ++j) gsum = X::dot2(G[j], ones, gsum);
        }
#pragma unroll
        for (int i = 0; i < IPT; ++i) {
            const int dy = dy0 + DYS * i;
            if (dy < KS) {  // (the same for all lanes of a wave where D >= 64)
                const uint32_t* row = vcur + (ty + dy) * ROW;
                uint32_t E[ROW], O[ROW - 1];  // pairs starting at even / at odd tokens
#pragma unroll
                for (int j = 0; j < ROW; ++j) E[j] = row[j];
#pragma unroll
                for (int j = 0; j + 1 < ROW; ++j) O[j] = __builtin_amdgcn_alignbit(E[j + 1], E[j], 16);
                // (consecutive dot products go to different accumulators: no chain of dependent ones)
#pragma unroll
                for (int pr = 0; pr < kApplyTW / 2; ++pr)
#pragma unroll
                    for (int dx = 0; dx < KS; ++dx)
                        acc[i][dx] = X::dot2(G[pr], (dx % 2) ? O[pr + dx / 2] : E[pr + dx / 2], acc[i][dx]);
            }
            __builtin_amdgcn_sched_barrier(0);  // one row in registers at a time
        }
        if constexpr (DB) {
            if (tile + p.chunks < p.n_tiles) {
#pragma unroll
                for (int k = 0; k < PIECES; ++k)
                    store_piece16(img + (buf ^ 1) * L::IMAGE, tid + NTHR * k, pre[k]);
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    // the four tile rows of a tap meet in LDS, in order
    __syncthreads();
    float* sums = reinterpret_cast<float*>(lds_raw);  // [NT][D]
#pragma unroll 1
    for (int ph = 0; ph < 4; ++ph) {
        if (ty == ph) {
#pragma unroll
            for (int i = 0; i < IPT; ++i) {
                const int dy = dy0 + DYS * i;
                if (dy < KS) {
#pragma unroll
                    for (int dx = 0; dx < KS; ++dx) {
                        float* s = sums + (dy * KS + dx) * D + c;
                        *s = ph == 0 ? acc[i][dx] : *s + acc[i][dx];
                    }
                }
            }
            if (dy0 == 0) {
                float* s = sums + KS * KS * D + c;
                *s = ph == 0 ? gsum : *s + gsum;
            }
        }
        __syncthreads();
    }
    float* o = part_out + (static_cast<size_t>(unit) * p.chunks + blockIdx.x) * NT * D;
    for (int idx = tid; idx < NT * D; idx += NTHR) o[idx] = sums[idx];
}

// grid = (ceil(heads * d * (taps + 1) / 16)), block = 256: sums the partial filter gradients over
// the batch and the chunks into dw [heads][d][taps] and dbias [heads][d] (may be null).  part:
// [B * heads][chunks][taps + 1][D].  Thread (slice, out) = (tid / 16, tid % 16): the 16 slices
// take runs of the (batch, chunk) pairs, each in order; slice 0 adds the slice sums in order (a
// fixed order of additions).
__global__ __launch_bounds__(256) void bwd_filter_combine_kernel(const float* __restrict__ part,
                                                                 float* __restrict__ dw,
                                                                 float* __restrict__ dbias, int B,
                                                                 int heads, int d, int D, int taps,
                                                                 int chunks)
{
    __shared__ float red[256];
    const int tid = threadIdx.x;
    const int i = blockIdx.x * 16 + tid % 16, sl = tid / 16;
    const int nt = taps + 1;
    const bool live = i < heads * d * nt;
    const int ch = i % d, e = (i / d) % nt, h = i / (nt * d);  // neighbours read neighbours
    const int items = B * chunks;  // (batch, chunk) pairs, batch-major
    const int per = (items + 15) / 16;
    float s = 0.f;
    if (live) {
        const int m1 = items < (sl + 1) * per ? items : (sl + 1) * per;
#pragma unroll 4
        for (int m = sl * per; m < m1; ++m) {
            const int b = m / chunks, k = m % chunks;
            s += part[((static_cast<size_t>(b) * heads + h) * chunks + k) * nt * D + e * D + ch];
        }
    }
    red[tid] = s;
    __syncthreads();
    if (sl == 0 && live) {
        for (int k = 1; k < 16; ++k) s += red[k * 16 + tid];
        if (e < taps) dw[(static_cast<size_t>(h) * d + ch) * taps + e] = s;
        else if (dbias) dbias[h * d + ch] = s;
    }
}

}  // namespace castling
