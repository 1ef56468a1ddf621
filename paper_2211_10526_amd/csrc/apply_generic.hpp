// Pass 2 on the vector ALU (any dtype): normalise Q per token, apply the state
// (Eq. 3 with the linear terms of Eq. 8), add the depthwise convolution of V
// over the token grid (DWConv term of Eq. 9), store.  fp32 products; with 16-bit I/O the
// linear branch runs on two-element dot products of 16-bit pairs.
#pragma once

#include "common.hpp"
#include "formats.hpp"

namespace castling {

struct ApplyParams {
    int N, grid_h, grid_w;
    int tiles_x;     // tiles per grid row
    int norm_none;   // 1: no denominator (literal Eq. 9)
    int do_linear;   // branch mask
    int do_dwconv;
    float eps;
    TensorStrides in, out;  // of q and v; of out
    // 1: `state` holds one final state per unit.  > 1: it holds that many partial states per
    // unit ([unit][split][StateLayout::SIZE], as pass 1 leaves them); the block sums them in
    // index order while it loads them (small problems: saves the combine launch)
    int n_partials;
    int d_valid;  // features per head in memory (<= D: narrower heads are padded with zeros)
    // Downsampling layers (pooled queries, Sec. 3.1): grid_h x grid_w above is the grid of the
    // queries and of out, q has strides of its own, and query (y, x) stands at position
    // (S*y, S*x) of the vgrid_h x vgrid_w grid of V (S = the kernel's stride; S = 1: same grid).
    TensorStrides qs;
    int vgrid_h, vgrid_w;
    int residual_q;  // 1: the query as stored is added to the result (residual connection)
    float lin_scale; // factor on the linear branch where there is no normaliser (1 in the forward)
};

constexpr int kApplyTH = 4;   // tile rows
constexpr int kApplyTW = 16;  // tile columns
constexpr int kApplyTokens = kApplyTH * kApplyTW;
constexpr int kQtStride = kApplyTokens + 4;  // floats; keeps float4 rows aligned

// Dynamic LDS the kernel needs, in bytes.
template <typename T, int D, int KS, int S = 1>
constexpr size_t apply_generic_lds_bytes()
{
    using L = StateLayout<D>;
    // fp32: state and q_hat in fp32.  16-bit: both as pairs of 16-bit values (see the kernel)
    const size_t phase_a =
        sizeof(T) == 4 ? sizeof(float) * (L::SIZE + D * kQtStride)
                       : 4 * (static_cast<size_t>(D / 2) * D + D / 2 + D + (D / 2) * kQtStride + kApplyTokens);
    const size_t halo = sizeof(T) * (S * (kApplyTH - 1) + KS) * (S * (kApplyTW - 1) + KS) * D;
    const size_t phase_b = ((halo + 15) / 16) * 16 + sizeof(float) * KS * KS * D;
    return phase_a > phase_b ? phase_a : phase_b;
}

// The 256 threads of a block compute one 4 x 16 tile (index `tile`, row-major over the tiles of
// the grid) of unit `unit`; thread (tt, tj) = (tid / 16, tid % 16) owns tokens
// (row tt/4, columns 4*(tt%4)..+3) and channels tj*D/16..+D/16-1.  `state`: the unit's state
// record(s), see ApplyParams::n_partials (global memory or LDS).  lds_raw: the block's dynamic
// LDS of apply_generic_lds_bytes<T, D, KS, S>() bytes.  S: stride of the queries on the grid of V.
template <typename T, int D, int KS, int S = 1>
__device__ __forceinline__ void apply_generic_tile(const T* __restrict__ q, const T* __restrict__ v,
                                                   const T* __restrict__ w,
                                                   const T* __restrict__ bias, const float* state,
                                                   T* __restrict__ out, int heads,
                                                   const ApplyParams& p, int unit, int tile,
                                                   unsigned char* lds_raw)
{
    constexpr int VEC = IO<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int RJ = D / 16;  // channels per thread
    constexpr int RAD = KS / 2;
    constexpr int HH = S * (kApplyTH - 1) + KS;  // halo tile rows
    constexpr int HW = S * (kApplyTW - 1) + KS;  // halo tile columns
    using L = StateLayout<D>;

    const int tid = threadIdx.x;
    const int head = unit % heads;
    const int ty0 = (tile / p.tiles_x) * kApplyTH;
    const int tx0 = (tile % p.tiles_x) * kApplyTW;
    const int tt = tid / 16, tj = tid % 16;
    const int my_row = tt / 4, my_col0 = (tt % 4) * 4;
    const long long in_off = unit_offset(unit, heads, p.in);
    const long long q_off = unit_offset(unit, heads, p.qs);
    const long long out_off = unit_offset(unit, heads, p.out);

    float res[4][RJ];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int j = 0; j < RJ; ++j) res[t][j] = 0.f;

    // The halo tile of V and the filters are needed after the linear branch only.  Where a thread
    // holds few pieces of them, their loads go out now and overlap it; on small problems (a
    // handful of blocks) the kernel is a chain of memory latencies otherwise.
    constexpr int HALO_PIECES = (HH * HW * LPR + 255) / 256;
    constexpr int W_PIECES = (D * KS * KS + 255) / 256;
    constexpr bool kPrefetch = HALO_PIECES <= 8 && W_PIECES <= 4;
    uint4 halo_pre[kPrefetch ? HALO_PIECES : 1];
    T w_pre[kPrefetch ? W_PIECES : 1];
    auto halo_piece = [&](int idx) {
        const int tok = idx / LPR, part = idx % LPR;
        const int y = S * ty0 - RAD + tok / HW, x = S * tx0 - RAD + tok % HW;
        uint4 val = make_uint4(0u, 0u, 0u, 0u);
        if (idx < HH * HW * LPR && part * VEC < p.d_valid && y >= 0 && y < p.vgrid_h && x >= 0 &&
            x < p.vgrid_w)
            val = *reinterpret_cast<const uint4*>(
                v + in_off + (static_cast<long long>(y) * p.vgrid_w + x) * p.in.n + part * VEC);
        return val;
    };
    if constexpr (kPrefetch) {
        if (p.do_dwconv) {
#pragma unroll
            for (int i = 0; i < HALO_PIECES; ++i) halo_pre[i] = halo_piece(tid + 256 * i);
            const T* wh = w + static_cast<size_t>(head) * p.d_valid * KS * KS;
#pragma unroll
            for (int i = 0; i < W_PIECES; ++i) {
                const int idx = tid + 256 * i;
                w_pre[i] = idx < p.d_valid * KS * KS ? wh[idx] : T{};
            }
        }
    }

    // ---------------------------------------------------------------- linear branch
    if (p.do_linear) {
        if constexpr (std::is_same<T, float>::value) {
            float* st = reinterpret_cast<float*>(lds_raw);  // state, pre-scaled
            float* qt = st + L::SIZE;                       // q_hat transposed: [D][kQtStride]
            const float* gs = state;
            if (p.n_partials == 1) {
                block_stage<L::SIZE, float>(
                    tid, [&](int i) { return gs[i]; },
                    [&](int i, float s) { st[i] = s * (i < L::VSUM ? kInvPi : 0.5f); });
            } else {
                for (int i = tid; i < L::SIZE; i += 256)
                    st[i] = sum_partials(gs + i, p.n_partials, L::SIZE) * (i < L::VSUM ? kInvPi : 0.5f);
            }

            constexpr int ROWS = 256 / LPR;  // token rows one pass of the block loads
            constexpr int PASSES = (kApplyTokens + ROWS - 1) / ROWS;
            const int lcol = (tid % LPR) * VEC;
    #pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int tl = pass * ROWS + tid / LPR;
                if (tl >= kApplyTokens) break;  // narrow rows: fewer threads than 256 are needed
                const int y = ty0 + tl / kApplyTW, x = tx0 + tl % kApplyTW;
                float qx[VEC];
                if (y < p.grid_h && x < p.grid_w && lcol < p.d_valid) {
                    IO<T>::load16(q + q_off + (static_cast<long long>(y) * p.grid_w + x) * p.qs.n + lcol, qx);
                } else {
    #pragma unroll
                    for (int e = 0; e < VEC; ++e) qx[e] = 0.f;
                }
                float ss = 0.f;
    #pragma unroll
                for (int e = 0; e < VEC; ++e) ss += qx[e] * qx[e];
                ss = group_sum<LPR>(ss);
                const float inv = 1.0f / fmaxf(sqrtf(ss), p.eps);
    #pragma unroll
                for (int e = 0; e < VEC; ++e) qt[(lcol + e) * kQtStride + tl] = qx[e] * inv;
            }
            __syncthreads();

            float den[4] = {0.f, 0.f, 0.f, 0.f};
    #pragma unroll 4
            for (int i = 0; i < D; ++i) {
                const float4 a4 = *reinterpret_cast<const float4*>(qt + i * kQtStride + tt * 4);
                const float a[4] = {a4.x, a4.y, a4.z, a4.w};
                const float ksi = st[L::KSUM + i];
                float b[RJ];
    #pragma unroll
                for (int j = 0; j < RJ; ++j) b[j] = st[L::S + i * D + tj * RJ + j];
    #pragma unroll
                for (int t = 0; t < 4; ++t) {
                    den[t] = fmaf(a[t], ksi, den[t]);
    #pragma unroll
                    for (int j = 0; j < RJ; ++j) res[t][j] = fmaf(a[t], b[j], res[t][j]);
                }
            }
    #pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float rden = p.norm_none ? p.lin_scale : 1.0f / (0.5f * static_cast<float>(p.N) + den[t]);
    #pragma unroll
                for (int j = 0; j < RJ; ++j) res[t][j] = (st[L::VSUM + tj * RJ + j] + res[t][j]) * rden;
            }
            __syncthreads();  // LDS is reused below
        } else {
            // 16-bit I/O: the products run as two-element dot products on pairs of 16-bit values,
            // q as stored (exact) against S / pi and ksum / pi rounded once to the I/O format --
            // the numerics of the matrix-core kernels -- and the per-token 1 / |q| multiplies
            // the fp32 sums afterwards.  Half the multiplies and half the LDS traffic of the
            // fp32 form.
            using X = typename std::conditional<std::is_same<T, f16_t>::value, F16Fmt, Bf16Fmt>::type;
            uint32_t* st2 = reinterpret_cast<uint32_t*>(lds_raw);   // [D/2][D]: (S[2i][j], S[2i+1][j])
            uint32_t* ks2 = st2 + (D / 2) * D;                      // [D/2]: pairs of ksum
            float* vh = reinterpret_cast<float*>(ks2 + D / 2);      // [D]: vsum / 2
            uint32_t* qt2 = reinterpret_cast<uint32_t*>(vh + D);    // [D/2][kQtStride]: pairs of q
            float* invl = reinterpret_cast<float*>(qt2 + (D / 2) * kQtStride);  // [tokens]: 1 / |q|
            const float tscale = X::table_scale(p.N), unsc = X::table_unscale(p.N);
            const float* gs = state;
            auto entry = [&](int i) {
                return p.n_partials == 1 ? gs[i] : sum_partials(gs + i, p.n_partials, L::SIZE);
            };
            if (p.n_partials == 1) {
                block_stage<(D / 2) * D, float2>(
                    tid,
                    [&](int idx) {
                        const int ip = idx / D, j = idx % D;
                        return make_float2(gs[L::S + (2 * ip) * D + j], gs[L::S + (2 * ip + 1) * D + j]);
                    },
                    [&](int idx, float2 s) { st2[idx] = X::pack(s.x * tscale, s.y * tscale); });
            } else {
                for (int idx = tid; idx < (D / 2) * D; idx += 256) {
                    const int ip = idx / D, j = idx % D;
                    st2[idx] = X::pack(entry(L::S + (2 * ip) * D + j) * tscale,
                                       entry(L::S + (2 * ip + 1) * D + j) * tscale);
                }
            }
            for (int idx = tid; idx < D / 2; idx += 256)
                ks2[idx] = X::pack(entry(L::KSUM + 2 * idx) * tscale, entry(L::KSUM + 2 * idx + 1) * tscale);
            for (int idx = tid; idx < D; idx += 256) vh[idx] = 0.5f * entry(L::VSUM + idx);

            constexpr int ROWS = 256 / LPR;  // token rows one pass of the block loads
            constexpr int PASSES = (kApplyTokens + ROWS - 1) / ROWS;
            const int lcol = (tid % LPR) * VEC;
#pragma unroll
            for (int pass = 0; pass < PASSES; ++pass) {
                const int tl = pass * ROWS + tid / LPR;
                if (tl >= kApplyTokens) break;  // narrow rows: fewer threads than 256 are needed
                const int y = ty0 + tl / kApplyTW, x = tx0 + tl % kApplyTW;
                uint4 raw = make_uint4(0u, 0u, 0u, 0u);
                if (y < p.grid_h && x < p.grid_w && lcol < p.d_valid)
                    raw = *reinterpret_cast<const uint4*>(
                        q + q_off + (static_cast<long long>(y) * p.grid_w + x) * p.qs.n + lcol);
                const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) ss = X::dot2(rw[e], rw[e], ss);
                ss = group_sum<LPR>(ss);
#pragma unroll
                for (int e = 0; e < 4; ++e) qt2[(lcol / 2 + e) * kQtStride + tl] = rw[e];
                if (tid % LPR == 0) invl[tl] = 1.0f / fmaxf(sqrtf(ss), p.eps);
            }
            __syncthreads();

            float den[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int ip = 0; ip < D / 2; ++ip) {
                const uint4 a4 = *reinterpret_cast<const uint4*>(qt2 + ip * kQtStride + tt * 4);
                const uint32_t aw[4] = {a4.x, a4.y, a4.z, a4.w};
                const uint32_t ksp = ks2[ip];
                uint32_t bw[RJ];
#pragma unroll
                for (int j = 0; j < RJ; ++j) bw[j] = st2[ip * D + tj * RJ + j];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    den[t] = X::dot2(aw[t], ksp, den[t]);
#pragma unroll
                    for (int j = 0; j < RJ; ++j) res[t][j] = X::dot2(aw[t], bw[j], res[t][j]);
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float inv = invl[tt * 4 + t] * unsc;
                const float rden =
                    p.norm_none ? p.lin_scale : 1.0f / (0.5f * static_cast<float>(p.N) + inv * den[t]);
#pragma unroll
                for (int j = 0; j < RJ; ++j) res[t][j] = (vh[tj * RJ + j] + inv * res[t][j]) * rden;
            }
            __syncthreads();  // LDS is reused below
        }
    }

    // ---------------------------------------------------------------- DWConv branch
    if (p.do_dwconv) {
        T* vh = reinterpret_cast<T*>(lds_raw);  // [HH][HW][D], zero outside the grid
        constexpr size_t halo_bytes = ((sizeof(T) * HH * HW * D + 15) / 16) * 16;
        float* wt = reinterpret_cast<float*>(lds_raw + halo_bytes);  // [KS*KS][D]

        if constexpr (kPrefetch) {
#pragma unroll
            for (int i = 0; i < HALO_PIECES; ++i) {
                const int idx = tid + 256 * i;
                if (idx < HH * HW * LPR)
                    *reinterpret_cast<uint4*>(vh + static_cast<size_t>(idx / LPR) * D + (idx % LPR) * VEC) =
                        halo_pre[i];
            }
#pragma unroll
            for (int i = 0; i < W_PIECES; ++i) {
                const int idx = tid + 256 * i;  // (w_pre is zero past the head's d_valid channels)
                if (idx < D * KS * KS)
                    wt[(idx % (KS * KS)) * D + idx / (KS * KS)] = IO<T>::to_f32(w_pre[i]);
            }
        } else {
            // (the loads of a thread go out in batches: see block_stage)
            block_stage<HH * HW * LPR, uint4, 256, 8>(
                tid, [&](int idx) { return halo_piece(idx); },
                [&](int idx, uint4 val) {
                    *reinterpret_cast<uint4*>(vh + static_cast<size_t>(idx / LPR) * D + (idx % LPR) * VEC) = val;
                });
            const T* wh = w + static_cast<size_t>(head) * p.d_valid * KS * KS;
            block_stage<D * KS * KS, T, 256, 8>(
                tid, [&](int idx) { return idx / (KS * KS) < p.d_valid ? wh[idx] : T{}; },
                [&](int idx, T val) {
                    wt[(idx % (KS * KS)) * D + idx / (KS * KS)] = IO<T>::to_f32(val);
                });
        }
        __syncthreads();

        float dw[4][RJ];
#pragma unroll
        for (int j = 0; j < RJ; ++j) {
            const int ch = tj * RJ + j;
            const float b0 = (bias && ch < p.d_valid) ? IO<T>::to_f32(bias[head * p.d_valid + ch]) : 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) dw[t][j] = b0;
        }
#pragma unroll 1
        for (int dy = 0; dy < KS; ++dy) {
            float wr[KS][RJ];
#pragma unroll
            for (int dx = 0; dx < KS; ++dx)
#pragma unroll
                for (int j = 0; j < RJ; ++j) wr[dx][j] = wt[(dy * KS + dx) * D + tj * RJ + j];
            const T* row = vh + (static_cast<size_t>(S * my_row + dy) * HW + S * my_col0) * D + tj * RJ;
#pragma unroll
            for (int xx = 0; xx < KS + 3 * S; ++xx) {
                float vin[RJ];
#pragma unroll
                for (int j = 0; j < RJ; ++j) vin[j] = IO<T>::to_f32(row[xx * D + j]);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int dx = xx - S * t;
                    if (dx >= 0 && dx < KS) {
#pragma unroll
                        for (int j = 0; j < RJ; ++j) dw[t][j] = fmaf(wr[dx][j], vin[j], dw[t][j]);
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < RJ; ++j) res[t][j] += dw[t][j];
    }

    // ---------------------------------------------------------------- store
    const int y = ty0 + my_row;
    if (y < p.grid_h) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int x = tx0 + my_col0 + t;
            if (x < p.grid_w && tj * RJ < p.d_valid) {  // (d_valid is a multiple of the piece)
                T* o = out + out_off + (static_cast<long long>(y) * p.grid_w + x) * p.out.n + tj * RJ;
                __attribute__((aligned(16))) T tmp[RJ];
                if (p.residual_q) {
                    const T* qr = q + q_off + (static_cast<long long>(y) * p.grid_w + x) * p.qs.n + tj * RJ;
#pragma unroll
                    for (int j = 0; j < RJ; ++j) res[t][j] += IO<T>::to_f32(qr[j]);
                }
#pragma unroll
                for (int j = 0; j < RJ; ++j) tmp[j] = IO<T>::from_f32(res[t][j]);
                constexpr int BYTES = sizeof(T) * RJ;
                if constexpr (BYTES % 16 == 0) {
#pragma unroll
                    for (int c = 0; c < BYTES / 16; ++c)
                        reinterpret_cast<uint4*>(o)[c] = reinterpret_cast<const uint4*>(tmp)[c];
                } else if constexpr (BYTES == 8) {
                    *reinterpret_cast<uint2*>(o) = *reinterpret_cast<const uint2*>(tmp);
                } else if constexpr (BYTES == 4) {
                    *reinterpret_cast<uint32_t*>(o) = *reinterpret_cast<const uint32_t*>(tmp);
                } else {
                    static_assert(BYTES == 2, "output piece of one thread");
                    *o = tmp[0];
                }
            }
        }
    }
}

// grid = (tiles_x * tiles_y, units), block = 256, dynamic LDS = apply_generic_lds_bytes.
template <typename T, int D, int KS, int S = 1>
__global__ __launch_bounds__(256) void apply_generic_kernel(const T* __restrict__ q,
                                                             const T* __restrict__ v,
                                                             const T* __restrict__ w,
                                                             const T* __restrict__ bias,
                                                             const float* __restrict__ state,
                                                             T* __restrict__ out, int heads,
                                                             ApplyParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int unit = blockIdx.y;
    apply_generic_tile<T, D, KS, S>(q, v, w, bias,
                                 state + static_cast<size_t>(unit) * p.n_partials * StateLayout<D>::SIZE,
                                 out, heads, p, unit, blockIdx.x, lds_raw);
}

// grid = (ceil(rows * D / 8 / 256), units), block = 256: zero the first `rows` token rows of every
// unit of out (16-byte pieces).  For tokens off the grid when only the DWConv branch is asked for.
template <typename T>
__global__ __launch_bounds__(256) void zero_rows_kernel(T* __restrict__ out, int rows, int d,
                                                        int heads, TensorStrides st)
{
    constexpr int VEC = IO<T>::VEC;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int per_row = d / VEC;
    if (i >= rows * per_row) return;
    T* o = out + unit_offset(blockIdx.y, heads, st) + (i / per_row) * st.n + (i % per_row) * VEC;
    *reinterpret_cast<uint4*>(o) = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace castling
