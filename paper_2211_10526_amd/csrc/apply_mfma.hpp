// Pass 2 for bf16 I/O, d = 64, on the matrix cores.
//
//   linear branch  (Eq. 3 with the linear terms of Eq. 8): q . S as a dense
//       16x16x32 bf16 MFMA per 16 tokens, per-token scalars on the vector ALU;
//   DWConv branch  (DWConv term of Eq. 9): a depthwise k x k filter is a banded
//       Toeplitz product along x.  v_mfma_f32_4x4x4_16b_bf16 multiplies 16
//       independent 4x4 blocks per instruction, one block per channel:
//           out[4 x][4 quads] += T_dy,m[4 x][4 x'] * V[4 x'][4 quads]
//       with T built from the filter row dy and V a run of 4 consecutive tokens
//       of one channel.  The linear branch enters as the C operand, so the sum of
//       Eq. 9 costs nothing.
//
// A block owns a strip of 16 grid columns x R rows of one (batch, head) unit.
// Wave c owns channels 16c..16c+15 for the DWConv and row (4s + c) of every
// 4-row step for the linear branch.  V rows enter LDS once, transposed to
// [quad][channel][4 tokens]; every wave keeps a sliding window of MFMA operands
// in registers, so each staged row is read from LDS once per wave.
#pragma once

#include "common.hpp"
#include "reduce_mfma.hpp"

namespace castling {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct ApplyMfmaParams {
    int N, grid_h, grid_w;
    int strips;     // 16-column strips per grid row
    int band_rows;  // output rows per block (multiple of 4)
    int norm_none, do_linear, do_dwconv;
    float eps;
};

constexpr int kStripW = 16;
constexpr int kVtQuadStride = 672;  // bytes per (row, quad) line: 8 octets * 80 B + pad
constexpr int kVtOctetStride = 80;  // 8 channels * 8 B + pad
constexpr int kVtRowStride = 6 * kVtQuadStride;
constexpr int kVtBytes = 4 * kVtRowStride;
constexpr int kLinTokPitch = 20;    // floats per (row, channel) line: 16 tokens + pad
constexpr int kLinBytes = 4 * 64 * kLinTokPitch * 4;
constexpr int kApplyMfmaLdsBytes = 2 * (kVtBytes + kLinBytes);

// Fragment tables prepared once per forward (see prepare kernels below):
//   sfrag [unit][nt 4][ks 2][lane 64] 8 x bf16 : S[i][j] / pi, i = 32 ks + 8 (lane/16) + e, j = 16 nt + lane%16
//   kfrag [unit][ks 2][lane 64]       8 x bf16 : ksum[i] / pi, same i, every column alike
//   vhalf [unit][64]                  fp32     : vsum[j] / 2
//   wfrag [head][c 4][dy KS][m 3][lane 64] 4 x bf16 : T[i][k] = w[ch][dy][4m - 4 + k - i + KS/2],
//          ch = 16 c + lane/4, i = lane%4, zero outside the filter
constexpr int kSfragPerUnit = 4 * 2 * 64 * 8;  // bf16 elements
constexpr int kKfragPerUnit = 2 * 64 * 8;

// grid = (ceil(units * 4096 / 2 / 256) ...) see launch; one thread sums the partials of
// two adjacent-i elements of S, writes the fp32 state and the bf16 fragment pair.
__global__ __launch_bounds__(256) void combine_frag_kernel(const float* __restrict__ partial,
                                                            float* __restrict__ state,
                                                            bf16_t* __restrict__ sfrag,
                                                            bf16_t* __restrict__ kfrag,
                                                            float* __restrict__ vhalf, int n_split)
{
    using L = StateLayout<64>;
    const int unit = blockIdx.y;
    const float* p = partial + static_cast<size_t>(unit) * n_split * L::SIZE;
    float* st = state + static_cast<size_t>(unit) * L::SIZE;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < 2048) {
        // S: t = ((nt*2 + ks)*64 + lane)*4 + e2
        const int e2 = t & 3, lane = (t >> 2) & 63, ks = (t >> 8) & 1, nt = t >> 9;
        const int i0 = 32 * ks + 8 * (lane >> 4) + 2 * e2;
        const int j = 16 * nt + (lane & 15);
        float s0 = 0.f, s1 = 0.f;
        for (int sp = 0; sp < n_split; ++sp) {
            s0 += p[static_cast<size_t>(sp) * L::SIZE + i0 * 64 + j];
            s1 += p[static_cast<size_t>(sp) * L::SIZE + (i0 + 1) * 64 + j];
        }
        st[i0 * 64 + j] = s0;
        st[(i0 + 1) * 64 + j] = s1;
        uint32_t* dst = reinterpret_cast<uint32_t*>(sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
        dst[t] = pack_bf16x2(s0 * kInvPi, s1 * kInvPi);
    } else if (t < 2048 + 128) {
        // column sums into the fp32 state; vsum / 2 for the apply kernel
        const int f = t - 2048;  // 0..63 ksum, 64..127 vsum
        float s = 0.f;
        for (int sp = 0; sp < n_split; ++sp) s += p[static_cast<size_t>(sp) * L::SIZE + L::KSUM + f];
        st[L::KSUM + f] = s;
        if (f >= 64) vhalf[unit * 64 + (f - 64)] = 0.5f * s;
    } else if (t < 2048 + 128 + 512) {
        // ksum fragments: t' = (ks*64 + lane)*4 + e2
        const int u = t - (2048 + 128);
        const int e2 = u & 3, lane = (u >> 2) & 63, ks = u >> 8;
        const int i0 = 32 * ks + 8 * (lane >> 4) + 2 * e2;
        float s0 = 0.f, s1 = 0.f;
        for (int sp = 0; sp < n_split; ++sp) {
            s0 += p[static_cast<size_t>(sp) * L::SIZE + L::KSUM + i0];
            s1 += p[static_cast<size_t>(sp) * L::SIZE + L::KSUM + i0 + 1];
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(kfrag + static_cast<size_t>(unit) * kKfragPerUnit);
        dst[u] = pack_bf16x2(s0 * kInvPi, s1 * kInvPi);
    }
}
constexpr int kCombineFragThreads = 2048 + 128 + 512;

// One thread per (head, c, dy, m, lane): the Toeplitz operand of the DWConv MFMA.
template <int KS>
__global__ __launch_bounds__(256) void dwconv_weight_frag_kernel(const bf16_t* __restrict__ w,
                                                                 bf16_t* __restrict__ wfrag,
                                                                 int heads)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= heads * 4 * KS * 3 * 64) return;
    const int lane = t & 63;
    const int m = (t >> 6) % 3;
    const int dy = (t / (64 * 3)) % KS;
    const int c = (t / (64 * 3 * KS)) & 3;
    const int head = t / (64 * 3 * KS * 4);
    const int ch = 16 * c + (lane >> 2), i = lane & 3;
    const bf16_t* wr = w + ((static_cast<size_t>(head) * 64 + ch) * KS + dy) * KS;
    bf16_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int dx = 4 * m - 4 + k - i + KS / 2;
        v[k] = (dx >= 0 && dx < KS) ? wr[dx] : static_cast<bf16_t>(0);
    }
    uint2 o;
    o.x = static_cast<uint32_t>(v[0]) | (static_cast<uint32_t>(v[1]) << 16);
    o.y = static_cast<uint32_t>(v[2]) | (static_cast<uint32_t>(v[3]) << 16);
    reinterpret_cast<uint2*>(wfrag)[t] = o;
}

// grid = (strips * bands, units), block = 256.
template <int KS>
__global__ __launch_bounds__(256) void apply_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ v, const bf16_t* __restrict__ bias,
    const bf16_t* __restrict__ sfrag, const bf16_t* __restrict__ kfrag,
    const float* __restrict__ vhalf, const bf16_t* __restrict__ wfrag, bf16_t* __restrict__ out,
    int heads, ApplyMfmaParams p)
{
    constexpr int D = 64;
    constexpr int RAD = KS / 2;
    constexpr int NCH = (KS + 3 + 3) / 4;  // 4-row chunks that cover the window
    constexpr int WR = 4 * NCH;            // window rows held in registers

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int c = tid >> 6;  // wave = channel group = row inside a step
    const int unit = blockIdx.y;
    const int head = unit % heads;
    const int strip = blockIdx.x % p.strips;
    const int band = blockIdx.x / p.strips;
    const int xs0 = strip * kStripW;
    const int y0 = band * p.band_rows;
    const int y_end = min(p.grid_h, y0 + p.band_rows);
    const int W = p.grid_w, H = p.grid_h;
    const size_t unit_off = static_cast<size_t>(unit) * p.N * D;
    const bf16_t* vu = v + unit_off;
    const bf16_t* qu = q + unit_off;

    auto vt_buf = [&](int b) { return lds + b * (kVtBytes + kLinBytes); };
    auto lin_buf = [&](int b) { return reinterpret_cast<float*>(lds + b * (kVtBytes + kLinBytes) + kVtBytes); };

    // ---- per-wave constants
    // DWConv lane roles: channel ch_dw, quad j (output x = xs0 + 4 j + i)
    const int blk = lane >> 2, j = lane & 3;
    const int ch_dw = 16 * c + blk;
    s16x4_t tw[KS][3];
    if (p.do_dwconv) {
        const uint2* wf = reinterpret_cast<const uint2*>(wfrag) +
                          ((static_cast<size_t>(head) * 4 + c) * KS * 3) * 64 + lane;
#pragma unroll
        for (int dy = 0; dy < KS; ++dy)
#pragma unroll
            for (int m = 0; m < 3; ++m) {
                const uint2 t = wf[(dy * 3 + m) * 64];
                tw[dy][m] = __builtin_bit_cast(s16x4_t, t);
            }
    }
    const float bias_dw = (bias && p.do_dwconv) ? bf16_to_f32(bias[head * D + ch_dw]) : 0.f;

    // linear lane roles: token tl (A operand row), feature group g; D layout: column n, tokens 4 g + r
    const int tl = lane & 15, g = lane >> 4;
    bf16x8_t sf[4][2], kf[2];
    float vh[4];
    if (p.do_linear) {
        const uint4* s4 = reinterpret_cast<const uint4*>(sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
        const uint4* k4 = reinterpret_cast<const uint4*>(kfrag + static_cast<size_t>(unit) * kKfragPerUnit);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                sf[nt][ks] = __builtin_bit_cast(bf16x8_t, s4[(nt * 2 + ks) * 64 + lane]);
            vh[nt] = vhalf[unit * D + 16 * nt + tl];
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) kf[ks] = __builtin_bit_cast(bf16x8_t, k4[ks * 64 + lane]);
    }

    // ---- cooperative V staging: 4 rows x 24 columns x 8 octets = 768 16-byte items
    uint4 vreg[3];
    auto load_v_rows = [&](int row_base) {
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int item = tid + 256 * it;
            const int r = item / 192, rem = item % 192;
            const int x = rem >> 3, oct = rem & 7;
            const int gy = row_base + r, gx = xs0 - 4 + x;
            vreg[it] = make_uint4(0u, 0u, 0u, 0u);
            if (gy >= 0 && gy < H && gx >= 0 && gx < W)
                vreg[it] = *reinterpret_cast<const uint4*>(vu + (static_cast<size_t>(gy) * W + gx) * D + oct * 8);
        }
    };
    auto write_v_rows = [&](unsigned char* vt) {
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int item = tid + 256 * it;
            const int r = item / 192, rem = item % 192;
            const int x = rem >> 3, oct = rem & 7;
            unsigned char* dst = vt + (r * 6 + (x >> 2)) * kVtQuadStride + oct * kVtOctetStride + (x & 3) * 2;
            const uint32_t wd[4] = {vreg[it].x, vreg[it].y, vreg[it].z, vreg[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                *reinterpret_cast<uint16_t*>(dst + (2 * e) * 8) = static_cast<uint16_t>(wd[e] & 0xffffu);
                *reinterpret_cast<uint16_t*>(dst + (2 * e + 1) * 8) = static_cast<uint16_t>(wd[e] >> 16);
            }
        }
    };

    // sliding window of DWConv data operands: win[idx][m], idx <-> input row (yo - RAD + idx)
    s16x4_t win[WR][3];
    auto read_window_rows = [&](const unsigned char* vt, int idx0) {
        const unsigned char* base = vt + (ch_dw >> 3) * kVtOctetStride + (ch_dw & 7) * 8;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int m = 0; m < 3; ++m) {
                const uint2 t = *reinterpret_cast<const uint2*>(base + (r * 6 + m + j) * kVtQuadStride);
                win[idx0 + r][m] = __builtin_bit_cast(s16x4_t, t);
            }
    };

    if (p.do_dwconv) {
#pragma unroll
        for (int chunk = 0; chunk < NCH; ++chunk) {
            load_v_rows(y0 - RAD + 4 * chunk);
            write_v_rows(vt_buf(0));
            __syncthreads();
            read_window_rows(vt_buf(0), 4 * chunk);
            __syncthreads();
        }
    }

    // ---- main loop over 4-row steps
    int buf = 0;
    for (int yo = y0; yo < y_end; yo += 4, buf ^= 1) {
        unsigned char* vt = vt_buf(buf);
        float* lin = lin_buf(buf);

        if (p.do_dwconv && yo > y0) {
            load_v_rows(yo - RAD + WR - 4);
            write_v_rows(vt);
        }

        // linear branch for row yo + c (all 64 channels of 16 tokens)
        if (p.do_linear) {
            const int y = yo + c, x = xs0 + tl;
            bf16x8_t a[2];
            a[0] = a[1] = __builtin_bit_cast(bf16x8_t, make_uint4(0u, 0u, 0u, 0u));
            if (y < H && x < W) {
                const uint4* src = reinterpret_cast<const uint4*>(qu + (static_cast<size_t>(y) * W + x) * D + 8 * g);
                a[0] = __builtin_bit_cast(bf16x8_t, src[0]);
                a[1] = __builtin_bit_cast(bf16x8_t, src[4]);
            }
            float ss = 0.f;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = static_cast<float>(a[ks][e]);
                    ss = fmaf(f, f, ss);
                }
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            f32x4_t acc[4], dk;
#pragma unroll
            for (int r = 0; r < 4; ++r) dk[r] = 0.f;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[nt][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], sf[nt][ks], acc[nt], 0, 0, 0);
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                dk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], kf[ks], dk, 0, 0, 0);
            float alpha[4], beta[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // |q|^2 of token 4 g + r lives in the lanes whose low four bits are that token
                const float ssr = __int_as_float(
                    __builtin_amdgcn_ds_bpermute((16 * g + 4 * g + r) * 4, __float_as_int(ss)));
                const float inv = 1.0f / fmaxf(sqrtf(ssr), p.eps);
                if (p.norm_none) {
                    alpha[r] = inv;
                    beta[r] = 1.0f;
                } else {
                    const float rden = 1.0f / (0.5f * static_cast<float>(p.N) + inv * dk[r]);
                    alpha[r] = inv * rden;
                    beta[r] = rden;
                }
            }
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                float4 o;
                o.x = fmaf(alpha[0], acc[nt][0], beta[0] * vh[nt]);
                o.y = fmaf(alpha[1], acc[nt][1], beta[1] * vh[nt]);
                o.z = fmaf(alpha[2], acc[nt][2], beta[2] * vh[nt]);
                o.w = fmaf(alpha[3], acc[nt][3], beta[3] * vh[nt]);
                *reinterpret_cast<float4*>(lin + ((c * 64 + 16 * nt + tl) * kLinTokPitch + 4 * g)) = o;
            }
        }
        __syncthreads();

        if (p.do_dwconv && yo > y0) {
            // slide the window down by four rows and take in the four new ones
#pragma unroll
            for (int idx = 0; idx < WR - 4; ++idx)
#pragma unroll
                for (int m = 0; m < 3; ++m) win[idx][m] = win[idx + 4][m];
            read_window_rows(vt, WR - 4);
        }

#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            f32x4_t acc;
            if (p.do_linear) {
                const float4 l4 = *reinterpret_cast<const float4*>(lin + ((rr * 64 + ch_dw) * kLinTokPitch + 4 * j));
                acc[0] = l4.x + bias_dw; acc[1] = l4.y + bias_dw; acc[2] = l4.z + bias_dw; acc[3] = l4.w + bias_dw;
            } else {
                acc[0] = acc[1] = acc[2] = acc[3] = bias_dw;
            }
            if (p.do_dwconv) {
#pragma unroll
                for (int dy = 0; dy < KS; ++dy)
#pragma unroll
                    for (int m = 0; m < 3; ++m)
                        acc = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(tw[dy][m], win[rr + dy][m], acc, 0, 0, 0);
            }
            const int y = yo + rr;
            if (y < y_end) {
                bf16_t* o = out + unit_off + (static_cast<size_t>(y) * W + xs0 + 4 * j) * D + ch_dw;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (xs0 + 4 * j + i < W) o[i * D] = f32_to_bf16(acc[i]);
            }
        }
    }
}

}  // namespace castling
