// Pass 1 for bf16 I/O on the matrix cores: K_hat^T V as a token-contraction on
// v_mfma_f32_32x32x16_bf16, the two column sums on the vector ALU.  Sec. 3.1
// (reassociation of kernel-based linear attention) and the sums of Eq. 3.
//
// Every wave streams its own slice of the block's tokens: 16-byte global loads
// (one token row = D/8 lanes), per-token 1/|k| with DPP adds, k_hat rounded to
// bf16 and staged with V in a wave-private LDS region in [token][feature] order,
// read back with the transposing LDS read so that each lane holds 8 consecutive
// tokens of one feature (the MFMA operand order), then MFMA.  No block barrier
// is needed inside the token loop.  The waves' accumulators are summed in a fixed
// tree through LDS, so the result does not depend on timing.
#pragma once

#include "common.hpp"
#include "formats.hpp"
#include "tables.hpp"

namespace castling {

constexpr int kReduceWaves = 4;
constexpr int kReduceIterTokens = 32;  // tokens one wave stages per iteration
constexpr int kReducePrefetch = 2;  // iterations whose loads are in flight

// One MFMA operand (8 consecutive tokens of one feature per lane) from a
// [token][feature] bf16 tile in LDS with `pitch` bytes per token row.
// tok0: first of the 16 tokens of this k-step; feat0: first of the 32 features.
__device__ __forceinline__ u32x4_t lds_operand_tr(const unsigned char* tile, int pitch, int tok0,
                                                   int feat0, int lane)
{
    const int g = lane >> 4, e = (lane >> 2) & 3, p = lane & 3;
    const int tok = tok0 + 8 * (g >> 1) + e;
    const int feat = feat0 + 16 * (g & 1) + 4 * p;
    const unsigned char* a = tile + tok * pitch + feat * 2;
    typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(a));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(a + 4 * pitch));
    s16x8_t r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(u32x4_t, r);
}

// Optional extra outputs of the reduce kernel.
//  - state != nullptr (only with n_split == 1 and D == 64): the block's result is final, so it
//    writes the fp32 state and the apply kernel's operand tables itself; no combine launch.
//  - w != nullptr: grid rows >= units build the DWConv weight operand table.
struct ReduceExtras {
    float* state;
    bf16_t* sfrag;
    bf16_t* kfrag;
    float* vhalf;
    const bf16_t* w;
    bf16_t* wfrag;
    int units, heads, ks;
    float tscale;  // table scale of the I/O format for this N
    uint32_t pair_skew;  // PAIR: bytes to add to the address of channels 32..63 of a token row
};

// grid = (n_split, units [+ weight rows]), block = 64 * kReduceWaves.  Same partial layout
// as the generic kernel: partial[u][s][StateLayout<D>::SIZE].
// PAIR (D = 64): a unit is two heads of 32 channels (whole 128-byte token rows when the heads
// are neighbours in memory); each half of a K row is normalised on its own, and of the 64 x 64
// product only the two diagonal 32 x 32 blocks mean anything.
template <int D, typename X, bool PAIR = false>
__global__ __launch_bounds__(64 * kReduceWaves) void reduce_mfma_kernel(
    const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, float* __restrict__ partial, int N,
    int n_split, int chunk, float eps, int heads, TensorStrides st, ReduceExtras ex)
{
    if (static_cast<int>(blockIdx.y) >= ex.units) {  // weight rows (uniform per block)
        const int row = blockIdx.y - ex.units;
        dwconv_weight_frag((row * gridDim.x + blockIdx.x) * (64 * kReduceWaves) + threadIdx.x, ex.w,
                           ex.wfrag, ex.heads, ex.ks);
        return;
    }
    constexpr int NW = kReduceWaves;
    constexpr int MT = D / 32;               // 32-wide tiles per side of S
    constexpr int LPR = D / 8;               // lanes per token row
    constexpr int TPL = 64 / LPR;            // tokens per wave-wide load
    constexpr int LOADS = kReduceIterTokens / TPL;
    constexpr int PITCH = D * 2 + 32;        // bytes per staged token row (bank spread)
    constexpr int TILE_BYTES = kReduceIterTokens * PITCH;
    constexpr int ACC_BYTES = MT * MT * 16 * 64 * 4;  // one wave's accumulators
    constexpr int STAGE_BYTES = NW * 2 * TILE_BYTES;
    constexpr int TREE_BYTES = (NW / 2) * ACC_BYTES;
    constexpr int SUMS_BYTES = NW * 64 * 16 * 4 + D * 4;  // + the block's final ksum
    constexpr int LDS_BYTES = (STAGE_BYTES > TREE_BYTES ? STAGE_BYTES : TREE_BYTES) >
                                      SUMS_BYTES
                                  ? (STAGE_BYTES > TREE_BYTES ? STAGE_BYTES : TREE_BYTES)
                                  : SUMS_BYTES;
    using L = StateLayout<D>;

    __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int unit = blockIdx.y;
    const int split = blockIdx.x;
    const int n_begin = split * chunk;
    const int n_end = min(N, n_begin + chunk);
    // each wave takes a contiguous slice, a multiple of the iteration size
    const int per_wave = ((chunk + NW * kReduceIterTokens - 1) / (NW * kReduceIterTokens)) *
                         kReduceIterTokens;
    const int w_begin = n_begin + wave * per_wave;
    const int w_end = min(n_end, w_begin + per_wave);

    const bf16_t* kb = k + unit_offset(unit, heads, st);
    const bf16_t* vb = v + unit_offset(unit, heads, st);
    const uint32_t tok_bytes = static_cast<uint32_t>(st.n) * 2;  // the host keeps N * tok_bytes below 4 GiB
    unsigned char* ks_tile = lds + wave * 2 * TILE_BYTES;
    unsigned char* vs_tile = ks_tile + TILE_BYTES;

    const int lrow = lane / LPR;         // token inside one wave-wide load
    const int lcol = (lane % LPR) * 8;   // first of this lane's 8 features

    f32x16_t acc[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    float ksum[8], vsum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ksum[e] = vsum[e] = 0.f;

    // software pipeline: the global loads of RPD iterations are in flight (see async_load16)
    constexpr int RPD = kReducePrefetch;
    static_assert(LOADS == 2 || LOADS == 4, "wait_async_loads takes 2 or 4 registers");
    u32x4_t kraw[RPD][LOADS], vraw[RPD][LOADS];
    const int n_iter = w_end > w_begin ? (w_end - w_begin + kReduceIterTokens - 1) / kReduceIterTokens : 0;
    const uint32_t lane_off = static_cast<uint32_t>(lcol * 2) + ((PAIR && lcol >= 32) ? ex.pair_skew : 0u);
    const float inv_eps = 1.0f / eps;
    const uint32_t one_lo = opaque_u32(X::kOneLo), one_hi = opaque_u32(X::kOneHi);

    // rows past the slice are loaded from a clamped (valid) address and zeroed when used
    auto issue_loads = [&](auto slot_c, int n0) {
        constexpr int slot = decltype(slot_c)::value;
        uint32_t off[LOADS];
#pragma unroll
        for (int j = 0; j < LOADS; ++j)
            off[j] = static_cast<uint32_t>(min(n0 + j * TPL + lrow, N - 1)) * tok_bytes + lane_off;
        // all K loads first, then all V loads: process() waits for them in this order
#pragma unroll
        for (int j = 0; j < LOADS; ++j) async_load16_stream(kraw[slot][j], kb, off[j]);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) async_load16(vraw[slot][j], vb, off[j]);
    };

    // ahead: iterations whose loads were issued after this slot's (fewer near the end)
    auto process = [&](auto slot_c, int n0, int ahead) {
        constexpr int slot = decltype(slot_c)::value;
        static_for<RPD>([&](auto a_c) {
            constexpr int Y = decltype(a_c)::value * 2 * LOADS;
            if (ahead == decltype(a_c)::value) {
                if constexpr (LOADS == 4) {
                    wait_async_loads<Y + LOADS>(kraw[slot][0], kraw[slot][1], kraw[slot][2], kraw[slot][3]);
                    wait_async_loads<Y>(vraw[slot][0], vraw[slot][1], vraw[slot][2], vraw[slot][3]);
                } else {
                    wait_async_loads<Y + LOADS>(kraw[slot][0], kraw[slot][1]);
                    wait_async_loads<Y>(vraw[slot][0], vraw[slot][1]);
                }
            }
        });
        // normalise, accumulate the column sums, stage k_hat and v
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const bool in = n0 + j * TPL + lrow < w_end;
            const u32x4_t zero = {0u, 0u, 0u, 0u};
            const u32x4_t kw = in ? kraw[slot][j] : zero;
            const u32x4_t vw = in ? vraw[slot][j] : zero;
            float kf[8];
            float ss = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kf[2 * i] = X::lo(kw[i]);
                kf[2 * i + 1] = X::hi(kw[i]);
                // two-element dot products on the raw pairs: |k|^2 two terms at a time, and the
                // V column sums without a conversion (the other half meets a zero)
                ss = X::dot2(kw[i], kw[i], ss);
                vsum[2 * i] = X::dot2(vw[i], one_lo, vsum[2 * i]);
                vsum[2 * i + 1] = X::dot2(vw[i], one_hi, vsum[2 * i + 1]);
            }
            ss = row_group_sum<PAIR ? LPR / 2 : LPR>(ss);
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
            const int row = j * TPL + lrow;
            *reinterpret_cast<u32x4_t*>(ks_tile + row * PITCH + lcol * 2) = kh;
            *reinterpret_cast<u32x4_t*>(vs_tile + row * PITCH + lcol * 2) = vw;
        }
        // LDS operations of one wave complete in issue order, and the staging tiles are
        // private to this wave: the reads below see the writes above without a barrier.
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s = 0; s < kReduceIterTokens / 16; ++s) {
            u32x4_t a[MT], b[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                a[t] = lds_operand_tr(ks_tile, PITCH, 16 * s, 32 * t, lane);
                b[t] = lds_operand_tr(vs_tile, PITCH, 16 * s, 32 * t, lane);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
                    acc[mt][nt] = X::mfma32(a[mt], b[nt], acc[mt][nt]);
        }
        __builtin_amdgcn_wave_barrier();
    };

    static_for<RPD>([&](auto slot) {
        if (decltype(slot)::value < n_iter)
            issue_loads(slot, w_begin + decltype(slot)::value * kReduceIterTokens);
    });
    for (int it = 0; it < n_iter; it += RPD) {
        static_for<RPD>([&](auto slot) {
            const int i = it + decltype(slot)::value;
            if (i < n_iter) {
                const int n0 = w_begin + i * kReduceIterTokens;
                process(slot, n0, min(RPD - 1, n_iter - 1 - i));
                if (i + RPD < n_iter) issue_loads(slot, n0 + RPD * kReduceIterTokens);
            }
        });
    }

    // ---- column sums: every lane's 16 partial sums go through LDS, summed in lane order
    __syncthreads();  // staging tiles are dead from here on
    {
        float* sums = reinterpret_cast<float*>(lds);  // [wave][lane][16]
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            sums[(wave * 64 + lane) * 16 + e] = ksum[e];
            sums[(wave * 64 + lane) * 16 + 8 + e] = vsum[e];
        }
        __syncthreads();
        float* out = partial + (static_cast<size_t>(unit) * n_split + split) * L::SIZE;
        if (tid < 2 * D) {
            const int which = tid / D;          // 0: ksum, 1: vsum
            const int f = tid % D;              // feature
            const int lc = f / 8, e = f % 8;    // lanes with lane % LPR == lc hold it
            float s = 0.f;
            for (int w = 0; w < NW; ++w)
                for (int r = 0; r < TPL; ++r)
                    s += sums[(w * 64 + r * LPR + lc) * 16 + which * 8 + e];
            out[(which ? L::VSUM : L::KSUM) + f] = s;
            if constexpr (D == 64) {
                if (ex.state) {  // final result: fp32 state, vsum / 2, and ksum kept for the table below
                    ex.state[static_cast<size_t>(unit) * L::SIZE + (which ? L::VSUM : L::KSUM) + f] = s;
                    if (which) ex.vhalf[unit * 64 + f] = 0.5f * s;
                    else sums[NW * 64 * 16 + f] = s;
                }
            }
        }
        __syncthreads();
        if constexpr (D == 64) {
            if (ex.state) {
                // ksum operand table: entry (ks, lane, e2) holds ksum[32 ks + 8 (lane / 16) + 2 e2 .. +1] * scale
                uint32_t* dst = reinterpret_cast<uint32_t*>(ex.kfrag + static_cast<size_t>(unit) * kKfragPerUnit);
                for (int u = tid; u < kKfragPerUnit / 2; u += 64 * NW) {
                    const int e2 = u & 3, fl = (u >> 2) & 63, ks = u >> 8;
                    const int i0 = 32 * ks + 8 * (fl >> 4) + 2 * e2;
                    dst[u] = X::pack(sums[NW * 64 * 16 + i0] * ex.tscale, sums[NW * 64 * 16 + i0 + 1] * ex.tscale);
                }
                __syncthreads();
            }
        }
    }

    // ---- K_hat^T V: fixed tree over the waves, (w0 + w2) + (w1 + w3)
    {
        // [slot][tile][register quad][lane] x 4 floats: 16-byte LDS accesses, lanes contiguous
        f32x4_t* tree = reinterpret_cast<f32x4_t*>(lds);
        constexpr int SLOT = MT * MT * 4 * 64;  // float4 per slot
#pragma unroll
        for (int half = NW / 2; half >= 1; half >>= 1) {
            if (wave >= half && wave < 2 * half) {
                f32x4_t* dst = tree + (wave - half) * SLOT + lane;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            f32x4_t q4;
#pragma unroll
                            for (int e = 0; e < 4; ++e) q4[e] = acc[mt][nt][4 * r4 + e];
                            dst[((mt * MT + nt) * 4 + r4) * 64] = q4;
                        }
            }
            __syncthreads();
            if (wave < half) {
                const f32x4_t* src = tree + wave * SLOT + lane;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const f32x4_t q4 = src[((mt * MT + nt) * 4 + r4) * 64];
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[mt][nt][4 * r4 + e] += q4[e];
                        }
            }
            __syncthreads();
        }
        if (wave == 0) {
            float* out = partial + (static_cast<size_t>(unit) * n_split + split) * L::SIZE + L::S;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int i = 32 * mt + (r / 4) * 8 + (lane / 32) * 4 + (r % 4);
                        const int j = 32 * nt + (lane % 32);
                        out[i * D + j] = acc[mt][nt][r];
                    }
            if constexpr (D == 64) {
                if (ex.state) {
                    // final result: fp32 state and the S operand table (16-bit pairs of S * scale)
                    float* st = ex.state + static_cast<size_t>(unit) * L::SIZE + L::S;
                    uint32_t* sf = reinterpret_cast<uint32_t*>(ex.sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int i = 32 * mt + (r / 4) * 8 + (lane / 32) * 4 + (r % 4);
                                const int j = 32 * nt + (lane % 32);
                                st[i * D + j] = acc[mt][nt][r];
                                if ((r & 1) == 0) {
                                    // table entry ((j/16)*2 + i/32, lane' = ((i%32)/8)*16 + j%16, (i%8)/2)
                                    const int t = (((j >> 4) * 2 + (i >> 5)) * 64 + (((i & 31) >> 3) * 16 + (j & 15))) * 4 +
                                                  ((i & 7) >> 1);
                                    sf[t] = X::pack(acc[mt][nt][r] * ex.tscale, acc[mt][nt][r + 1] * ex.tscale);
                                }
                            }
                }
            }
        }
    }
}

}  // namespace castling
