// Operand tables that pass 1 (or the combine) prepares for the matrix-core apply kernel.
#pragma once

#include "common.hpp"

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

}  // namespace castling
