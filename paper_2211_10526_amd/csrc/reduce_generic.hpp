// Pass 1 on the vector ALU (any dtype): normalise K per token and reduce over a
// chunk of tokens to a partial state (K_hat^T V, K_hat column sum, V column sum),
// then a fixed-order combine of the partials.  fp32 products; with 16-bit I/O and heads of
// 64 channels or more, two-element dot products on pairs of tokens.  Sec. 3.1 (reassociation of
// kernel-based linear attention) and the sums of Eq. 3 of the paper.
#pragma once

#include "common.hpp"
#include "formats.hpp"

namespace castling {

// This thread's 16 raw bytes of token row n, features lcol .. (zeros for n >= n_end and for
// features >= d_valid: heads narrower than the kernel's width are padded with zero features).
template <typename T>
__device__ __forceinline__ uint4 load_row_piece(const T* base, int n, int n_end, long long tok_stride,
                                                int lcol, int d_valid)
{
    return (n < n_end && lcol < d_valid) ? *reinterpret_cast<const uint4*>(base + n * tok_stride + lcol)
                                         : make_uint4(0u, 0u, 0u, 0u);
}

// Tokens per LDS tile of the reduce loop (256 threads, 16 bytes each).
template <typename T, int D>
constexpr int reduce_generic_tile() { return 256 / (D / IO<T>::VEC); }

// Register tiling of S = K_hat^T V: a thread owns an R x R block, (D / R)^2 threads cover S, and
// the block's 256 threads form G such groups that take the tokens of a tile in turn (a 4 x 4
// block needs one 16-byte LDS read per operand and token; with the whole block on one copy of
// S, narrow heads would read LDS once per multiply).  Their sums meet in LDS in group order.
template <int D>
struct ReduceTiling {
    static constexpr int R = D / 16 > 4 ? D / 16 : 4;
    static constexpr int SIDE = D / R;
    static constexpr int GROUP = SIDE * SIDE;  // threads per copy of S
    static constexpr int G = 256 / GROUP;
    static constexpr int RED_FLOATS = G > 1 ? G * StateLayout<D>::SIZE : 1;
    static_assert(GROUP * G == 256, "head width");
};

// The 256 threads of a block reduce tokens [n_begin, n_end) of the unit whose K and V start
// at kb, vb to one state record at `out` (StateLayout<D>; global memory or LDS).  kh, vv:
// two LDS tiles of [reduce_generic_tile][D] floats; red: ReduceTiling<D>::RED_FLOATS floats.
template <typename T, int D>
__device__ __forceinline__ void reduce_generic_tokens(const T* __restrict__ kb,
                                                      const T* __restrict__ vb, int n_begin,
                                                      int n_end, long long tok_stride, float eps,
                                                      float* out, float (*kh)[D], float (*vv)[D],
                                                      float* red, int d_valid)
{
    constexpr int VEC = IO<T>::VEC;  // elements per 16-byte load
    constexpr int LPR = D / VEC;     // lanes that share one token row
    constexpr int TILE = 256 / LPR;  // tokens staged per iteration
    using RT = ReduceTiling<D>;
    // 16-bit I/O and wide heads: products on pairs of tokens (below); narrow heads do too little
    // arithmetic per staged row to pay for the 2-byte LDS writes of that form
    constexpr bool kPairs = sizeof(T) == 2 && D >= 64;
    constexpr int R = RT::R, G = RT::G;
    using L = StateLayout<D>;

    const int tid = threadIdx.x;
    const int grp = tid / RT::GROUP, ti = (tid % RT::GROUP) / RT::SIDE, tj = tid % RT::SIDE;
    const int lrow = tid / LPR, lcol = (tid % LPR) * VEC;

    float acc[R][R];
    float ks[R], vs[R];
#pragma unroll
    for (int a = 0; a < R; ++a) {
        ks[a] = 0.f;
        vs[a] = 0.f;
#pragma unroll
        for (int b = 0; b < R; ++b) acc[a][b] = 0.f;
    }

    // the rows of the next tile are loaded while this one is multiplied: with few tokens per
    // block the loop is a chain of memory latencies otherwise
    uint4 kraw = load_row_piece(kb, n_begin + lrow, n_end, tok_stride, lcol, d_valid);
    uint4 vraw = load_row_piece(vb, n_begin + lrow, n_end, tok_stride, lcol, d_valid);
    uint32_t ones = 0u;  // (1, 1) in the 16-bit format
    if constexpr (kPairs) {
        using X = typename std::conditional<std::is_same<T, f16_t>::value, F16Fmt, Bf16Fmt>::type;
        ones = opaque_u32(X::kOneLo | X::kOneHi);
    }
    for (int n0 = n_begin; n0 < n_end; n0 += TILE) {
        float kx[VEC], vx[VEC];
        const uint4 vraw_cur = vraw;
        IO<T>::widen16(kraw, kx);
        IO<T>::widen16(vraw, vx);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) ss += kx[e] * kx[e];
        ss = group_sum<LPR>(ss);
        const float inv = 1.0f / fmaxf(sqrtf(ss), eps);

        __syncthreads();  // the previous tile has been consumed
        if constexpr (!kPairs) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                kh[lrow][lcol + e] = kx[e] * inv;
                vv[lrow][lcol + e] = vx[e];
            }
        } else {
            // 16-bit I/O: the tiles hold pairs of consecutive tokens, k_hat rounded once to the
            // I/O format (as the matrix-core kernels round it) in the half its token has in
            // the pair; the products below then take two tokens per instruction
            T* kh16 = reinterpret_cast<T*>(&kh[0][0]) + ((lrow >> 1) * D + lcol) * 2 + (lrow & 1);
            T* vv16 = reinterpret_cast<T*>(&vv[0][0]) + ((lrow >> 1) * D + lcol) * 2 + (lrow & 1);
            const T* vsrc = reinterpret_cast<const T*>(&vraw_cur);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                kh16[2 * e] = IO<T>::from_f32(kx[e] * inv);
                vv16[2 * e] = vsrc[e];
            }
        }
        kraw = load_row_piece(kb, n0 + TILE + lrow, n_end, tok_stride, lcol, d_valid);  // (zeros past the end)
        vraw = load_row_piece(vb, n0 + TILE + lrow, n_end, tok_stride, lcol, d_valid);
        __syncthreads();

        if constexpr (!kPairs) {
            static_assert(TILE % G == 0, "every group takes the same number of tokens of a tile");
#pragma unroll 4
            for (int t = grp; t < TILE; t += G) {
                float a[R], b[R];
#pragma unroll
                for (int e = 0; e < R; ++e) {
                    a[e] = kh[t][ti * R + e];
                    b[e] = vv[t][tj * R + e];
                }
#pragma unroll
                for (int x = 0; x < R; ++x) {
#pragma unroll
                    for (int y = 0; y < R; ++y) acc[x][y] = fmaf(a[x], b[y], acc[x][y]);
                    ks[x] += a[x];
                    vs[x] += b[x];
                }
            }
        } else {
            using X = typename std::conditional<std::is_same<T, f16_t>::value, F16Fmt, Bf16Fmt>::type;
            static_assert((TILE / 2) % G == 0, "every group takes the same number of token pairs");
            const uint32_t* kh2 = reinterpret_cast<const uint32_t*>(&kh[0][0]);
            const uint32_t* vv2 = reinterpret_cast<const uint32_t*>(&vv[0][0]);
#pragma unroll 4
            for (int tp = grp; tp < TILE / 2; tp += G) {
                uint32_t a[R], b[R];
#pragma unroll
                for (int e = 0; e < R; ++e) {
                    a[e] = kh2[tp * D + ti * R + e];
                    b[e] = vv2[tp * D + tj * R + e];
                }
#pragma unroll
                for (int x = 0; x < R; ++x) {
#pragma unroll
                    for (int y = 0; y < R; ++y) acc[x][y] = X::dot2(a[x], b[y], acc[x][y]);
                    ks[x] = X::dot2(a[x], ones, ks[x]);
                    vs[x] = X::dot2(b[x], ones, vs[x]);
                }
            }
        }
    }

    // this group's sums: straight to `out` if it is the only one, else through LDS
    float* mine = G > 1 ? red + grp * L::SIZE : out;
#pragma unroll
    for (int x = 0; x < R; ++x)
#pragma unroll
        for (int y = 0; y < R; ++y) mine[L::S + (ti * R + x) * D + tj * R + y] = acc[x][y];
    if (tj == 0)
#pragma unroll
        for (int x = 0; x < R; ++x) mine[L::KSUM + ti * R + x] = ks[x];
    if (ti == 0)
#pragma unroll
        for (int x = 0; x < R; ++x) mine[L::VSUM + tj * R + x] = vs[x];
    if constexpr (G > 1) {
        __syncthreads();
        for (int i = tid; i < L::SIZE; i += 256) {
            float s = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) s += red[g * L::SIZE + i];
            out[i] = s;
        }
    }
}

// grid = (n_split, units), block = 256.
// Block (s, u) reduces tokens [s*chunk, min(N, (s+1)*chunk)) of unit u and writes
// partial[u][s][StateLayout<D>::SIZE].  d_valid <= D: features per head in memory.
template <typename T, int D>
__global__ __launch_bounds__(256) void reduce_generic_kernel(const T* __restrict__ k,
                                                              const T* __restrict__ v,
                                                              float* __restrict__ partial, int N,
                                                              int n_split, int chunk, float eps,
                                                              int heads, TensorStrides st, int d_valid)
{
    constexpr int TILE = reduce_generic_tile<T, D>();
    using L = StateLayout<D>;
    __shared__ __attribute__((aligned(16))) float kh[TILE][D];
    __shared__ __attribute__((aligned(16))) float vv[TILE][D];
    __shared__ __attribute__((aligned(16))) float red[ReduceTiling<D>::RED_FLOATS];
    const int unit = blockIdx.y, split = blockIdx.x;
    const int n_begin = split * chunk;
    const long long off = unit_offset(unit, heads, st);
    reduce_generic_tokens<T, D>(k + off, v + off, n_begin, min(N, n_begin + chunk), st.n, eps,
                                partial + (static_cast<size_t>(unit) * n_split + split) * L::SIZE,
                                kh, vv, red, d_valid);
}

// grid = (ceil(SIZE/256), units), block = 256.  state[u][i] = sum over splits in
// index order: the order never depends on which block finished first.
template <int D>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ partial,
                                                       float* __restrict__ state, int n_split)
{
    using L = StateLayout<D>;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int unit = blockIdx.y;
    if (i >= L::SIZE) return;
    const float* p = partial + static_cast<size_t>(unit) * n_split * L::SIZE + i;
    state[static_cast<size_t>(unit) * L::SIZE + i] = sum_partials(p, n_split, L::SIZE);
}

}  // namespace castling
