// Operand tables that pass 1 (or the combine) prepares for the matrix-core apply kernel, and
// the kernels that build them.
#pragma once

#include "common.hpp"
#include "formats.hpp"

namespace castling {

// Fragment tables prepared once per forward:
//   sfrag [unit][nt 4][ks 2][lane 64] 8 x bf16 : S[i][j] / pi, i = 32 ks + 8 (lane/16) + e, j = 16 nt + lane%16
//   kfrag [unit][ks 2][lane 64]       8 x bf16 : ksum[i] / pi, same i, every column alike
//   vhalf [unit][64]                  fp32     : vsum[j] / 2
//   wfrag [head][c 4][dy KS][m 3][lane 64] 4 x bf16 : T[i][k] = w[ch][dy][4m - 4 + k - i + KS/2],
//          ch = 16 c + lane/4, i = lane%4, zero outside the filter
constexpr int kSfragPerUnit = 4 * 2 * 64 * 8;  // bf16 elements
constexpr int kKfragPerUnit = 2 * 64 * 8;

// Thread t of heads * 4 * ks * 3 * 64 builds one 8-byte entry of wfrag: the Toeplitz operand
// of the DWConv MFMA for (head, c, dy, m, lane).
__device__ __forceinline__ void dwconv_weight_frag(int t, const bf16_t* __restrict__ w,
                                                   bf16_t* __restrict__ wfrag, int heads, int ks)
{
    if (t >= heads * 4 * ks * 3 * 64) return;
    const int lane = t & 63;
    const int m = (t >> 6) % 3;
    const int dy = (t / (64 * 3)) % ks;
    const int c = (t / (64 * 3 * ks)) & 3;
    const int head = t / (64 * 3 * ks * 4);
    const int ch = 16 * c + (lane >> 2), i = lane & 3;
    const bf16_t* wr = w + ((static_cast<size_t>(head) * 64 + ch) * ks + dy) * ks;
    bf16_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int dx = 4 * m - 4 + k - i + ks / 2;
        const int dxc = min(max(dx, 0), ks - 1);
        const bf16_t val = wr[dxc];
        v[k] = (dx == dxc) ? val : static_cast<bf16_t>(0);
    }
    uint2 o;
    o.x = static_cast<uint32_t>(v[0]) | (static_cast<uint32_t>(v[1]) << 16);
    o.y = static_cast<uint32_t>(v[2]) | (static_cast<uint32_t>(v[3]) << 16);
    reinterpret_cast<uint2*>(wfrag)[t] = o;
}

// grid = (ceil(kCombineFragThreads / 256), units + weight_rows).  Rows < units: fixed-order
// sum of the partial states of one unit; writes the fp32 state and the bf16 MFMA operand
// tables of the apply kernel.  Rows >= units (only when w != nullptr): the DWConv weight
// operand table, so that a whole forward needs no separate launch for it.
template <typename X>
__global__ __launch_bounds__(256) void combine_frag_kernel(
    const float* __restrict__ partial, float* __restrict__ state, bf16_t* __restrict__ sfrag,
    bf16_t* __restrict__ kfrag, float* __restrict__ vhalf, int n_split, int units,
    const bf16_t* __restrict__ w, bf16_t* __restrict__ wfrag, int heads, int ks, float tscale)
{
    using L = StateLayout<64>;
    if (static_cast<int>(blockIdx.y) >= units) {
        const int row = blockIdx.y - units;
        dwconv_weight_frag((row * gridDim.x + blockIdx.x) * 256 + threadIdx.x, w, wfrag, heads, ks);
        return;
    }
    const int unit = blockIdx.y;
    const float* p = partial + static_cast<size_t>(unit) * n_split * L::SIZE;
    float* st = state + static_cast<size_t>(unit) * L::SIZE;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < 2048) {
        // S: t = ((nt*2 + ks)*64 + lane)*4 + e2
        const int e2 = t & 3, lane = (t >> 2) & 63, ks = (t >> 8) & 1, nt = t >> 9;
        const int i0 = 32 * ks + 8 * (lane >> 4) + 2 * e2;
        const int j = 16 * nt + (lane & 15);
        const float s0 = sum_partials(p + i0 * 64 + j, n_split, L::SIZE);
        const float s1 = sum_partials(p + (i0 + 1) * 64 + j, n_split, L::SIZE);
        st[i0 * 64 + j] = s0;
        st[(i0 + 1) * 64 + j] = s1;
        uint32_t* dst = reinterpret_cast<uint32_t*>(sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
        dst[t] = X::pack(s0 * tscale, s1 * tscale);
    } else if (t < 2048 + 128) {
        // column sums into the fp32 state; vsum / 2 for the apply kernel
        const int f = t - 2048;  // 0..63 ksum, 64..127 vsum
        const float s = sum_partials(p + L::KSUM + f, n_split, L::SIZE);
        st[L::KSUM + f] = s;
        if (f >= 64) vhalf[unit * 64 + (f - 64)] = 0.5f * s;
    } else if (t < 2048 + 128 + 512) {
        // ksum fragments: t' = (ks*64 + lane)*4 + e2
        const int u = t - (2048 + 128);
        const int e2 = u & 3, lane = (u >> 2) & 63, ks = u >> 8;
        const int i0 = 32 * ks + 8 * (lane >> 4) + 2 * e2;
        const float s0 = sum_partials(p + L::KSUM + i0, n_split, L::SIZE);
        const float s1 = sum_partials(p + L::KSUM + i0 + 1, n_split, L::SIZE);
        uint32_t* dst = reinterpret_cast<uint32_t*>(kfrag + static_cast<size_t>(unit) * kKfragPerUnit);
        dst[u] = X::pack(s0 * tscale, s1 * tscale);
    }
}
constexpr int kCombineFragThreads = 2048 + 128 + 512;

// The same for pairs of heads with d = 32 that pass 2 runs as one 64-channel unit: row `pu`
// sums the partials of the pair, writes the fp32 states of units 2 pu and 2 pu + 1
// (StateLayout<32>) and builds the pair's operand tables: S block diagonal (zero where row and
// column belong to different heads), ksum and vsum / 2 one head after the other.
// wide = 1: pass 1 ran on the pairs too (partials in StateLayout<64>, of whose S only the
// diagonal 32 x 32 blocks are read); wide = 0: on the single heads (StateLayout<32>).
template <typename X>
__global__ __launch_bounds__(256) void combine_pair_frag_kernel(
    const float* __restrict__ partial, float* __restrict__ state, bf16_t* __restrict__ sfrag,
    bf16_t* __restrict__ kfrag, float* __restrict__ vhalf, int n_split, int pairs, int wide,
    const bf16_t* __restrict__ w, bf16_t* __restrict__ wfrag, int pair_heads, int ks, float tscale)
{
    using L = StateLayout<32>;
    using P = StateLayout<64>;
    if (static_cast<int>(blockIdx.y) >= pairs) {
        const int row = blockIdx.y - pairs;
        dwconv_weight_frag((row * gridDim.x + blockIdx.x) * 256 + threadIdx.x, w, wfrag, pair_heads, ks);
        return;
    }
    const int pu = blockIdx.y;
    const int t = blockIdx.x * 256 + threadIdx.x;
    const size_t stride = wide ? P::SIZE : L::SIZE;
    // entry (i, j) of the pair's S (same head on both sides), entry f of its ksum (f < 64) or
    // vsum (f >= 64), summed over the splits
    auto s_entry = [&](int i, int j) {
        const float* p = wide ? partial + static_cast<size_t>(pu) * n_split * P::SIZE + i * 64 + j
                              : partial + static_cast<size_t>(2 * pu + (i >> 5)) * n_split * L::SIZE +
                                    (i & 31) * 32 + (j & 31);
        return sum_partials(p, n_split, stride);
    };
    auto v_entry = [&](int f) {
        const float* p = wide ? partial + static_cast<size_t>(pu) * n_split * P::SIZE + P::KSUM + f
                              : partial + static_cast<size_t>(2 * pu + ((f >> 5) & 1)) * n_split * L::SIZE +
                                    (f < 64 ? L::KSUM : L::VSUM) + (f & 31);
        return sum_partials(p, n_split, stride);
    };
    auto stat = [&](int head) { return state + static_cast<size_t>(2 * pu + head) * L::SIZE; };
    if (t < 2048) {
        // S: t = ((nt*2 + ks)*64 + lane)*4 + e2 over the pair's 64 x 64 table
        const int e2 = t & 3, lane = (t >> 2) & 63, kst = (t >> 8) & 1, nt = t >> 9;
        const int i0 = 32 * kst + 8 * (lane >> 4) + 2 * e2;
        const int j = 16 * nt + (lane & 15);
        uint32_t word = 0u;
        if ((i0 >> 5) == (j >> 5)) {
            const int head = i0 >> 5, li = i0 & 31, lj = j & 31;
            const float s0 = s_entry(i0, j), s1 = s_entry(i0 + 1, j);
            stat(head)[li * 32 + lj] = s0;
            stat(head)[(li + 1) * 32 + lj] = s1;
            word = X::pack(s0 * tscale, s1 * tscale);
        }
        reinterpret_cast<uint32_t*>(sfrag + static_cast<size_t>(pu) * kSfragPerUnit)[t] = word;
    } else if (t < 2048 + 128) {
        const int f = t - 2048;  // 0..63 ksum of the pair, 64..127 vsum of the pair
        const int head = (f >> 5) & 1, lf = f & 31;
        const float s = v_entry(f);
        stat(head)[(f < 64 ? L::KSUM : L::VSUM) + lf] = s;
        if (f >= 64) vhalf[pu * 64 + (f - 64)] = 0.5f * s;
    } else if (t < 2048 + 128 + 512) {
        const int u = t - (2048 + 128);
        const int e2 = u & 3, lane = (u >> 2) & 63, kst = u >> 8;
        const int i0 = 32 * kst + 8 * (lane >> 4) + 2 * e2;
        reinterpret_cast<uint32_t*>(kfrag + static_cast<size_t>(pu) * kKfragPerUnit)[u] =
            X::pack(v_entry(i0) * tscale, v_entry(i0 + 1) * tscale);
    }
}

__global__ __launch_bounds__(256) void dwconv_weight_frag_kernel(const bf16_t* __restrict__ w,
                                                                 bf16_t* __restrict__ wfrag,
                                                                 int heads, int ks)
{
    dwconv_weight_frag(blockIdx.x * 256 + threadIdx.x, w, wfrag, heads, ks);
}

}  // namespace castling
