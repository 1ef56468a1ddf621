// The whole layer in one kernel for units whose tokens fit on chip (bf16 or fp16, d = 64 or two
// neighbouring heads of d = 32, N <= 256, filter size <= 5): one block per unit loads K, V, Q
// once, builds the state K_hat^T V, sum k_hat, sum v on the matrix cores (Sec. 3.1
// reassociation, sums of Eq. 3), keeps it in LDS as MFMA operands, applies it to the unit's own
// queries (Eq. 3 with the linear terms of Eq. 8) and adds the depthwise convolution of V read
// from LDS (Eq. 9).  At these sizes the state (17 KB fp32 + 10 KB of operands per unit) is as
// large as a tensor of the unit (25 KB at N = 196), so keeping it on chip and launching once
// beats the two-pass path.
//
// Block = 4 waves, two blocks per compute unit.  The global loads are issued with inline
// global_load and explicit s_waitcnt vmcnt and consumed in issue order: K, V, filters and bias
// at the start, Q between the two iterations of phase 1.
//   phase 1  wave w normalises and stages tokens 64 w .. 64 w + 63 (V rows stay in LDS for
//            the convolution), accumulates K_hat^T V with v_mfma_f32_32x32x16;
//   between  column sums through lane shuffles; the four waves' 64 x 64 sums by recursive
//            halving, after which wave w owns quadrant w of S;
//   phase 2  S / pi (every wave its quadrant), ksum / pi, vsum / 2, filters and bias go to
//            LDS tables;
//   phase 3  per chunk of 64 tokens: wave w computes the linear branch of 16 tokens
//            (v_mfma_f32_16x16x32) into an fp32 LDS tile; then every thread adds the
//            convolution for 8 channels of two tokens with two-element dot products on the raw
//            16-bit pairs and stores 16 bytes per token, 8 lanes per 128-byte output line.
#pragma once

#include "apply_mfma.hpp"
#include "common.hpp"
#include "reduce_mfma.hpp"
#include "tables.hpp"

namespace castling {

constexpr int kFusedMaxTokens = 256;
constexpr int kFusedMaxKs = 5;
constexpr int kFusedPitch = 160;  // bytes per token row of the V and k_hat tiles (bank spread)
constexpr int kFusedVBytes = (kFusedMaxTokens + 1) * kFusedPitch;  // + one row of zeros
constexpr int kFusedKtileBytes = 32 * kFusedPitch;  // per wave
constexpr int kFusedLinPitch = 68;                  // floats per token row of the linear tile
// k_hat staging, then column-sum scratch, then the linear tile share one region
constexpr int kFusedUnionBytes = 4 * kFusedKtileBytes;
static_assert(kFusedUnionBytes >= 64 * kFusedLinPitch * 4, "linear tile");
static_assert(kFusedUnionBytes >= 4 * 64 * 16 * 4, "column-sum scratch");
constexpr int kFusedSfragOff = kFusedVBytes + kFusedUnionBytes;  // 4 x 2 x 64 x 16 bytes
constexpr int kFusedKfragOff = kFusedSfragOff + 8192;            // 2 x 64 x 16 bytes
constexpr int kFusedVhalfOff = kFusedKfragOff + 2048;            // 64 floats
constexpr int kFusedBiasOff = kFusedVhalfOff + 256;              // 64 floats
constexpr int kFusedWOff = kFusedBiasOff + 256;                  // [tap][channel] floats
constexpr int kFusedLdsBytes = kFusedWOff + kFusedMaxKs * kFusedMaxKs * 64 * 4;
// the reduction tree (2 slots of one wave's accumulators) overlays the union region and the
// tables behind it, all of which are written only after the tree
static_assert(kFusedVBytes + 2 * 16384 <= kFusedLdsBytes, "tree scratch");
static_assert(2 * kFusedLdsBytes <= 160 * 1024, "two blocks per compute unit");

struct FusedParams {
    int N, grid_h, grid_w;
    int extra;  // tokens in front of the grid: no convolution term
    int norm_none;
    float eps;
    TensorStrides in, out;
    uint32_t in_skew, out_skew;  // pairs of heads: bytes added to the address of channels 32..63 of a row (else 0)
};

// One 32 x 32 quadrant of a wave's accumulators to / from an exchange slot in LDS
// ([register quad][lane] float4: 16-byte accesses, lanes contiguous).  By value: the accumulators
// must stay in registers.
__device__ __forceinline__ void put_quadrant(f32x4_t* dst, f32x16_t t)
{
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        f32x4_t q4;
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) q4[e4] = t[4 * r4 + e4];
        dst[r4 * 64] = q4;
    }
}
__device__ __forceinline__ f32x16_t add_quadrant(const f32x4_t* src, f32x16_t t)
{
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4_t q4 = src[r4 * 64];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) t[4 * r4 + e4] += q4[e4];
    }
    return t;
}

// grid = (units), block = 256, dynamic LDS = kFusedLdsBytes.
// state: [units][StateLayout<64>::SIZE] fp32 copy of the state (nullptr = not wanted).
// PAIR: a unit is two neighbouring heads of 32 channels (see apply_mfma_kernel): each half of a
// K or q row has its own norm, row sum and 32 x 32 state; the S operand table is block diagonal
// and `state` takes two StateLayout<32> records per unit.
template <int KS, bool LIN, bool DW, typename X, bool PAIR = false>
__global__ __launch_bounds__(256, 2) void fused_small_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ w, const bf16_t* __restrict__ bias, float* __restrict__ state,
    bf16_t* __restrict__ out, int heads, FusedParams p)
{
    static_assert(KS <= kFusedMaxKs && (KS & 1), "filter size");
    constexpr int D = 64;
    constexpr int RAD = KS / 2;
    constexpr int PITCH = kFusedPitch;
    constexpr int LP = kFusedLinPitch;
    using L = StateLayout<D>;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char* const vtile = lds;
    unsigned char* const un = lds + kFusedVBytes;
    uint32_t* const wl = reinterpret_cast<uint32_t*>(lds + kFusedWOff);
    float* const bl = reinterpret_cast<float*>(lds + kFusedBiasOff);
    float* const vhalf = reinterpret_cast<float*>(lds + kFusedVhalfOff);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int unit = blockIdx.x;
    const int head = unit % heads;
    const int N = p.N, W = p.grid_w, H = p.grid_h;
    const uint32_t in_tok = static_cast<uint32_t>(p.in.n) * 2;
    const uint32_t out_tok = static_cast<uint32_t>(p.out.n) * 2;
    const long long in_off = unit_offset(unit, heads, p.in);
    const bf16_t* const qb = q + in_off;
    const bf16_t* const kb = k + in_off;
    const bf16_t* const vb = v + in_off;

    const int lrow = lane >> 3;        // token inside one wave-wide load of 8 token rows
    const int lcol = (lane & 7) * 8;   // first of this lane's 8 features
    const int tl = lane & 15, g = lane >> 4;

    // ---- every global load of the unit, in the order in which it is consumed.  Addresses
    // past the unit are clamped to valid ones, so each wave issues the same number of loads
    // and the counts below hold.
    constexpr int NK = LIN ? 4 : 0;          // K loads per iteration of 32 tokens
    constexpr int PER_IT = NK + 4;
    constexpr int NWB = DW ? 2 : 0;          // filters, bias
    constexpr int NQ = LIN ? 8 : 0;          // 2 per chunk of 64 tokens
    u32x4_t kraw[2][4], vraw[2][4], qraw[4][2], wraw, braw;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int n0 = 64 * wave + 32 * it;
        uint32_t off[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            off[j] = static_cast<uint32_t>(min(n0 + 8 * j + lrow, N - 1)) * in_tok + lcol * 2 +
                     (lcol >= 32 ? p.in_skew : 0u);
        if constexpr (LIN) {
#pragma unroll
            for (int j = 0; j < 4; ++j) async_load16_stream(kraw[it][j], kb, off[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) async_load16(vraw[it][j], vb, off[j]);
    }
    constexpr int W_CHUNKS = KS * KS * 8;  // 16-byte pieces of one head's filters
    if constexpr (DW) {
        const bf16_t* wh = w + static_cast<size_t>(head) * D * KS * KS;
        async_load16(wraw, wh, static_cast<uint32_t>(min(tid, W_CHUNKS - 1)) * 16);
        // without a bias the load still happens (from the filters) and its value is dropped
        const bf16_t* bh = bias ? bias + head * D : wh;
        async_load16(braw, bh, static_cast<uint32_t>(tid & 7) * 16);
    }
    // q is not needed before phase 3: its loads go out between the two iterations of phase 1,
    // where their issue overlaps the arithmetic of the other waves
    auto issue_q_loads = [&]() {
        if constexpr (LIN) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int tok = min(64 * c + 16 * wave + tl, N - 1);
                const uint32_t off = static_cast<uint32_t>(tok) * in_tok + g * 16;
                async_load16_stream(qraw[c][0], qb, off);
                async_load16_stream(qraw[c][1], qb, off + 64 + p.in_skew);
            }
        }
    };

    // the row of zeros behind the V tile: what a filter tap outside the grid reads
    if (tid < 8) {
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4_t*>(vtile + kFusedMaxTokens * PITCH + tid * 16) = zero;
    }
    // ---- phase 1: normalise K, stage k_hat and V, accumulate K_hat^T V
    f32x16_t acc[2][2];
    float ksum[8], vsum[8];
    if constexpr (LIN) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ksum[e] = vsum[e] = 0.f;
    }
    const float inv_eps = 1.0f / p.eps;
    const uint32_t one_lo = opaque_u32(X::kOneLo), one_hi = opaque_u32(X::kOneHi);
    const float tscale = X::table_scale(N), unsc = X::table_unscale(N);
    unsigned char* const ktile = un + wave * kFusedKtileBytes;

    static_for<2>([&](auto it_c) {
        constexpr int it = decltype(it_c)::value;
        // loads issued after this iteration's: the q loads go out after iteration 0
        constexpr int YOUNGER = it == 0 ? PER_IT + NWB : NWB + NQ;
        const int n0 = 64 * wave + 32 * it;
        if constexpr (LIN)
            wait_async_loads<YOUNGER + 4>(kraw[it][0], kraw[it][1], kraw[it][2], kraw[it][3]);
        wait_async_loads<YOUNGER>(vraw[it][0], vraw[it][1], vraw[it][2], vraw[it][3]);
        if (n0 >= N) {  // uniform per wave
            if constexpr (it == 0) issue_q_loads();
            return;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = 8 * j + lrow;
            const bool in = n0 + row < N;
            const u32x4_t zero = {0u, 0u, 0u, 0u};
            const u32x4_t vw = in ? vraw[it][j] : zero;
            *reinterpret_cast<u32x4_t*>(vtile + (n0 + row) * PITCH + lcol * 2) = vw;
            if constexpr (LIN) {
                const u32x4_t kw = in ? kraw[it][j] : zero;
                float kf[8];
                float ss = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kf[2 * i] = X::lo(kw[i]);
                    kf[2 * i + 1] = X::hi(kw[i]);
                    ss = X::dot2(kw[i], kw[i], ss);
                    vsum[2 * i] = X::dot2(vw[i], one_lo, vsum[2 * i]);
                    vsum[2 * i + 1] = X::dot2(vw[i], one_hi, vsum[2 * i + 1]);
                }
                ss = row_group_sum<PAIR ? 4 : 8>(ss);
                // 1 / max(|k|, eps) with the hardware reciprocal square root (1 ulp)
                const float inv = fminf(__builtin_amdgcn_rsqf(ss), inv_eps);
                u32x4_t kh;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = kf[2 * i] * inv, b = kf[2 * i + 1] * inv;
                    ksum[2 * i] += a;
                    ksum[2 * i + 1] += b;
                    kh[i] = X::pack(a, b);
                }
                *reinterpret_cast<u32x4_t*>(ktile + row * PITCH + lcol * 2) = kh;
            }
        }
        if constexpr (LIN) {
            // LDS operations of one wave complete in issue order; these 32 rows of both tiles
            // are written by this wave only
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                u32x4_t a[2], b[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    a[t] = lds_operand_tr(ktile, PITCH, 16 * s, 32 * t, lane);
                    b[t] = lds_operand_tr(vtile + n0 * PITCH, PITCH, 16 * s, 32 * t, lane);
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = X::mfma32(a[mt], b[nt], acc[mt][nt]);
            }
            __builtin_amdgcn_wave_barrier();
        }
        if constexpr (it == 0) issue_q_loads();
    });
    __syncthreads();  // V is staged; the k_hat tiles are dead

    // ---- between the passes: four block barriers.  Scratch, as byte offsets from `un`:
    //   [0, 32 KB)   exchange slots of the tree (round 1: 8 KB per wave, round 2: 4 KB per wave)
    //   [32 KB, +2K) per-wave column sums (inside the filter table, which is written last)
    //   [16 KB, +256) ksum in fp32, for the ksum operand table
    // The operand tables, vsum / 2, bias and filters lie inside the first 32 KB and behind it;
    // each is written only after the last read of the scratch it overlays.
    float colsum = 0.f;  // tid < 64: ksum[tid]; tid < 128: vsum[tid - 64]
    f32x4_t* const xch = reinterpret_cast<f32x4_t*>(un);
    float* const wsums = reinterpret_cast<float*>(un + 32768);
    float* const ksumf = reinterpret_cast<float*>(un + 16384);
    static_assert(kFusedVBytes + 32768 + 2048 <= kFusedLdsBytes, "per-wave column sums");
    static_assert(kFusedWOff - kFusedVBytes <= 32768, "column sums overlay the filter table only");
    // f(mt, nt) with the quadrant of S this wave ends up owning: wave = 2 mt + nt
    auto own_quadrant = [&](auto&& f) {
        static_for<4>([&](auto w_c) {
            constexpr int WV = decltype(w_c)::value;
            if (wave == WV)
                f(std::integral_constant<int, (WV >> 1)>{}, std::integral_constant<int, (WV & 1)>{});
        });
    };
    constexpr int QUAD = 4 * 64;  // float4 per quadrant of one wave

    if constexpr (LIN) {
        // column sums of the wave: lanes with equal lane % 8 hold the same features
#pragma unroll
        for (int e8 = 0; e8 < 8; ++e8) {
            float a = dpp_add<kDppRowRor8>(ksum[e8]), b = dpp_add<kDppRowRor8>(vsum[e8]);
            a += __shfl_xor(a, 16, 64);
            b += __shfl_xor(b, 16, 64);
            a += __shfl_xor(a, 32, 64);
            b += __shfl_xor(b, 32, 64);
            ksum[e8] = a;
            vsum[e8] = b;
        }
        if (lane < 8) {
#pragma unroll
            for (int e8 = 0; e8 < 8; ++e8) {
                wsums[(wave * 8 + lane) * 16 + e8] = ksum[e8];
                wsums[(wave * 8 + lane) * 16 + 8 + e8] = vsum[e8];
            }
        }
        // K_hat^T V: the four waves' 64 x 64 partial sums by recursive halving.  Round 1 pairs
        // wave w with w ^ 2: each sends the two quadrants of the other's half of the rows.
        own_quadrant([&](auto mt_c, auto) {
            constexpr int MT = decltype(mt_c)::value;
            f32x4_t* dst = xch + wave * 2 * QUAD + lane;
            put_quadrant(dst, acc[1 - MT][0]);
            put_quadrant(dst + QUAD, acc[1 - MT][1]);
        });
    }
    __syncthreads();
    if constexpr (LIN) {
        if (tid < 2 * D) {
            const int which = tid / D, f = tid % D;
            const int lc = f / 8, e8 = f % 8;
#pragma unroll
            for (int wv = 0; wv < 4; ++wv) colsum += wsums[(wv * 8 + lc) * 16 + which * 8 + e8];
            if (state) {
                if constexpr (PAIR) {
                    using L32 = StateLayout<32>;
                    state[static_cast<size_t>(2 * unit + (f >> 5)) * L32::SIZE +
                          (which ? L32::VSUM : L32::KSUM) + (f & 31)] = colsum;
                } else {
                    state[static_cast<size_t>(unit) * L::SIZE + (which ? L::VSUM : L::KSUM) + f] = colsum;
                }
            }
        }
        own_quadrant([&](auto mt_c, auto) {
            constexpr int MT = decltype(mt_c)::value;
            const f32x4_t* src = xch + (wave ^ 2) * 2 * QUAD + lane;
            acc[MT][0] = add_quadrant(src, acc[MT][0]);
            acc[MT][1] = add_quadrant(src + QUAD, acc[MT][1]);
        });
    }
    __syncthreads();
    if constexpr (LIN) {
        if (tid < D) ksumf[tid] = colsum;
        else if (tid < 2 * D) vhalf[tid - D] = 0.5f * colsum;
        // round 2 pairs wave w with w ^ 1: each sends the other's quadrant of its half
        own_quadrant([&](auto mt_c, auto nt_c) {
            constexpr int MT = decltype(mt_c)::value, NT = decltype(nt_c)::value;
            put_quadrant(xch + wave * QUAD + lane, acc[MT][1 - NT]);
        });
    }
    __syncthreads();
    // ---- phase 2: operand tables of the linear branch (same layouts as sfrag / kfrag), each
    // wave from its own quadrant; filters and bias
    if constexpr (LIN) {
        own_quadrant([&](auto mt_c, auto nt_c) {
            constexpr int MT = decltype(mt_c)::value, NT = decltype(nt_c)::value;
            // (w + w^2) + (w^1 + w^3)
            acc[MT][NT] = add_quadrant(xch + (wave ^ 1) * QUAD + lane, acc[MT][NT]);
            uint32_t* sf = reinterpret_cast<uint32_t*>(lds + kFusedSfragOff);
            // PAIR: the quadrants off the diagonal mix two heads; their table entries are zero
            constexpr bool kZero = PAIR && MT != NT;
            float* st = nullptr;
            if (state) {
                if constexpr (PAIR) st = state + static_cast<size_t>(2 * unit + MT) * StateLayout<32>::SIZE;
                else st = state + static_cast<size_t>(unit) * L::SIZE + L::S;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 32 * MT + (r / 4) * 8 + (lane / 32) * 4 + (r % 4);
                const int j = 32 * NT + (lane % 32);
                if constexpr (PAIR) {
                    if (st && !kZero) st[(i & 31) * 32 + (j & 31)] = acc[MT][NT][r];
                } else {
                    if (st) st[i * D + j] = acc[MT][NT][r];
                }
                if ((r & 1) == 0) {
                    const int t = (((j >> 4) * 2 + (i >> 5)) * 64 + (((i & 31) >> 3) * 16 + (j & 15))) * 4 +
                                  ((i & 7) >> 1);
                    sf[t] = kZero ? 0u : X::pack(acc[MT][NT][r] * tscale, acc[MT][NT][r + 1] * tscale);
                }
            }
        });
        uint32_t* kfr = reinterpret_cast<uint32_t*>(lds + kFusedKfragOff);
        for (int u = tid; u < kKfragPerUnit / 2; u += 256) {
            const int e2 = u & 3, fl = (u >> 2) & 63, ks = u >> 8;
            const int i0 = 32 * ks + 8 * (fl >> 4) + 2 * e2;
            kfr[u] = X::pack(ksumf[i0] * tscale, ksumf[i0 + 1] * tscale);
        }
    }
    if constexpr (DW) {
        // filters [channel][tap] -> LDS [tap][channel], one 32-bit word each: the 16-bit weight in
        // the half its channel has inside a pair of channels, zero in the other half (the
        // operand of the two-element dot product below); bias -> fp32
        wait_async_loads<NQ + 1>(wraw);
        if (tid < W_CHUNKS) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = 8 * tid + i;
                const uint32_t word = wraw[i >> 1];
                const uint32_t raw = (i & 1) ? (word >> 16) : (word & 0xffffu);
                const int ch = e / (KS * KS);
                wl[(e % (KS * KS)) * D + ch] = (ch & 1) ? (raw << 16) : raw;
            }
        }
        wait_async_loads<NQ>(braw);
        if (tid < 8) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t word = braw[i >> 1];
                const float val = (i & 1) ? X::hi(word) : X::lo(word);
                bl[8 * tid + i] = bias ? val : 0.f;
            }
        }
    }
    __syncthreads();

    // ---- phase 3
    u32x4_t sf[4][2], kf[2];
    float vh[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (LIN) {
        const uint4* s4 = reinterpret_cast<const uint4*>(lds + kFusedSfragOff);
        const uint4* k4 = reinterpret_cast<const uint4*>(lds + kFusedKfragOff);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                sf[nt][ks] = __builtin_bit_cast(u32x4_t, s4[(nt * 2 + ks) * 64 + lane]);
            vh[nt] = vhalf[16 * nt + tl];
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) kf[ks] = __builtin_bit_cast(u32x4_t, k4[ks * 64 + lane]);
    }
    const float half_n = 0.5f * static_cast<float>(N);
    float* const lin = reinterpret_cast<float*>(un);
    unsigned char* const ob = reinterpret_cast<unsigned char*>(out + unit_offset(unit, heads, p.out));
    const int oct = tid & 7;
    // this thread's 8 channels: bias, and for the small filters every tap, held in registers
    // (the LDS reads of the filters were two thirds of the convolution's LDS traffic)
    constexpr bool kRegW = DW && KS <= 3;
    float breg[8];
    uint32_t wreg[kRegW ? KS * KS * 8 : 1];
    if constexpr (DW) {
#pragma unroll
        for (int i = 0; i < 8; ++i) breg[i] = bl[8 * oct + i];
        if constexpr (kRegW) {
#pragma unroll
            for (int tap = 0; tap < KS * KS; ++tap) {
                const uint4 w0 = *reinterpret_cast<const uint4*>(wl + tap * D + 8 * oct);
                const uint4 w1 = *reinterpret_cast<const uint4*>(wl + tap * D + 8 * oct + 4);
                wreg[tap * 8 + 0] = w0.x; wreg[tap * 8 + 1] = w0.y;
                wreg[tap * 8 + 2] = w0.z; wreg[tap * 8 + 3] = w0.w;
                wreg[tap * 8 + 4] = w1.x; wreg[tap * 8 + 5] = w1.y;
                wreg[tap * 8 + 6] = w1.z; wreg[tap * 8 + 7] = w1.w;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) breg[i] = 0.f;
    }

    static_for<4>([&](auto c_c) {
        constexpr int c = decltype(c_c)::value;
        if (64 * c >= N) return;  // uniform per block
        if constexpr (LIN) {
            wait_async_loads<2 * (3 - c)>(qraw[c][0], qraw[c][1]);
            if (64 * c + 16 * wave < N) {  // uniform per wave
                const bool qok = 64 * c + 16 * wave + tl < N;
                const u32x4_t zero = {0u, 0u, 0u, 0u};
                u32x4_t a[2];
                a[0] = qok ? qraw[c][0] : zero;
                a[1] = qok ? qraw[c][1] : zero;
                // |q_t|^2 on the matrix cores: the diagonal of Q Q^T.  PAIR: k-step 0 holds the
                // first head's features and k-step 1 the second's; each gets its own products.
                constexpr int NH = PAIR ? 2 : 1;
                const f32x4_t z4 = {0.f, 0.f, 0.f, 0.f};
                f32x4_t gram[NH], dk[NH], ac[4];
                if constexpr (PAIR) {
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        gram[hh] = X::mfma16(a[hh], a[hh], z4);
                        dk[hh] = X::mfma16(a[hh], kf[hh], z4);
                    }
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) ac[nt] = X::mfma16(a[nt >> 1], sf[nt][nt >> 1], z4);
                } else {
                    gram[0] = dk[0] = z4;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        gram[0] = X::mfma16(a[ks], a[ks], gram[0]);
                        dk[0] = X::mfma16(a[ks], kf[ks], dk[0]);
                    }
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        ac[nt] = z4;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) ac[nt] = X::mfma16(a[ks], sf[nt][ks], ac[nt]);
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float alpha[NH], beta[NH];
#pragma unroll
                    for (int hh = 0; hh < NH; ++hh) {
                        // entry (m, m) of the Gram tile, m = 4 g + r, sits in lane 16 (m / 4) + m, register m % 4
                        const float ssr = __int_as_float(
                            __builtin_amdgcn_ds_bpermute((20 * g + r) * 4, __float_as_int(gram[hh][r])));
                        float inv = fminf(__builtin_amdgcn_rsqf(ssr), inv_eps);
                        if constexpr (X::kHalf) inv *= unsc;  // the tables are scaled down
                        if (p.norm_none) {
                            alpha[hh] = inv;
                            beta[hh] = 1.0f;
                        } else {
                            beta[hh] = __builtin_amdgcn_rcpf(half_n + inv * dk[hh][r]);
                            alpha[hh] = inv * beta[hh];
                        }
                    }
                    float* row = lin + (16 * wave + 4 * g + r) * LP + tl;
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        const int hh = PAIR ? (nt >> 1) : 0;
                        row[16 * nt] = fmaf(alpha[hh], ac[nt][r], beta[hh] * vh[nt]);
                    }
                }
            }
            __syncthreads();
        }
        // convolution, sum of Eq. 9 and store: item = (token, 8 channels); a thread has the two
        // tokens tid / 8 and tid / 8 + 32 of the chunk, and every filter tap serves both.
        // (Uniform per wave) a wave whose first token is past the end has none: the ragged
        // last chunk of N = 196 has work for one wave only.
        if (64 * c + 8 * wave < N) {
            const int tloc0 = tid >> 3;
            float o[2][8];
            int ty[2], tx[2];
            bool live[2], conv[2];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const int tloc = tloc0 + 32 * h2;
                const int t = 64 * c + tloc;
                live[h2] = t < N;
                conv[h2] = DW && live[h2] && t >= p.extra;
                const int tg = max(t - p.extra, 0);  // position on the grid
                ty[h2] = tg / W;
                tx[h2] = tg - ty[h2] * W;
                if constexpr (LIN) {
                    const float4 l0 = *reinterpret_cast<const float4*>(lin + tloc * LP + 8 * oct);
                    const float4 l1 = *reinterpret_cast<const float4*>(lin + tloc * LP + 8 * oct + 4);
                    o[h2][0] = l0.x; o[h2][1] = l0.y; o[h2][2] = l0.z; o[h2][3] = l0.w;
                    o[h2][4] = l1.x; o[h2][5] = l1.y; o[h2][6] = l1.z; o[h2][7] = l1.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) o[h2][i] = 0.f;
                }
                if (conv[h2]) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) o[h2][i] += breg[i];
                }
            }
            if constexpr (DW) {
                // per token: which filter rows and columns fall on the grid, and the LDS address of
                // the token's column in each of those rows; a tap off the grid reads the zero row
                bool rok[2][KS], cok[2][KS];
                int rbase[2][KS];
                const int zero_addr = kFusedMaxTokens * PITCH + oct * 16;
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
                    for (int dd = 0; dd < KS; ++dd) {
                        const int yy = ty[h2] + dd - RAD;
                        rok[h2][dd] = conv[h2] && static_cast<unsigned>(yy) < static_cast<unsigned>(H);
                        cok[h2][dd] = static_cast<unsigned>(tx[h2] + dd - RAD) < static_cast<unsigned>(W);
                        rbase[h2][dd] = (p.extra + yy * W + tx[h2]) * PITCH + oct * 16;
                    }
#pragma unroll kRegW ? KS : 1
                for (int dy = 0; dy < KS; ++dy) {
#pragma unroll
                    for (int dx = 0; dx < KS; ++dx) {
                        uint32_t wv[8];
                        if constexpr (kRegW) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) wv[i] = wreg[(dy * KS + dx) * 8 + i];
                        } else {
                            const uint32_t* wt = wl + (dy * KS + dx) * D + 8 * oct;
                            const uint4 w0 = *reinterpret_cast<const uint4*>(wt);
                            const uint4 w1 = *reinterpret_cast<const uint4*>(wt + 4);
                            wv[0] = w0.x; wv[1] = w0.y; wv[2] = w0.z; wv[3] = w0.w;
                            wv[4] = w1.x; wv[5] = w1.y; wv[6] = w1.z; wv[7] = w1.w;
                        }
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2) {
                            const bool ok = rok[h2][dy] && cok[h2][dx];
                            const int addr = ok ? rbase[h2][dy] + (dx - RAD) * PITCH : zero_addr;
                            const u32x4_t vw = *reinterpret_cast<const u32x4_t*>(vtile + addr);
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                // one instruction per channel, no conversion: the zero half of
                                // the weight word removes the pair's other channel
                                o[h2][2 * i] = X::dot2(vw[i], wv[2 * i], o[h2][2 * i]);
                                o[h2][2 * i + 1] = X::dot2(vw[i], wv[2 * i + 1], o[h2][2 * i + 1]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const int t = 64 * c + tloc0 + 32 * h2;
                if (live[h2])
                    store16_stream(ob + (static_cast<uint32_t>(t) * out_tok + oct * 16 +
                                         (oct >= 4 ? p.out_skew : 0u)),
                                   X::pack(o[h2][0], o[h2][1]), X::pack(o[h2][2], o[h2][3]),
                                   X::pack(o[h2][4], o[h2][5]), X::pack(o[h2][6], o[h2][7]));
            }
        }
        if constexpr (LIN) {
            if (64 * (c + 1) < N) __syncthreads();  // the next chunk overwrites the linear tile
        }
    });
    // loads that were never waited for (chunks past N) must land before the registers die
    if constexpr (LIN) wait_async_loads<0>(qraw[3][0], qraw[3][1]);
}

}  // namespace castling
