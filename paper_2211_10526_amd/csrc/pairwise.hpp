// O(N^2) attention on the matrix cores (bf16 or fp16, d = 64), the training-time companions of
// the linear-angular layer:
//   SPARSE   Mask_thr(Softmax(scale * A B^T)) V, the auxiliary branch of Eq. 10 (Sec. 3.2.2);
//            A, B are q, k or their unit rows; Mask_thr(x) = x if x > thr else 0.  The mask
//            applies to normalised probabilities, so the keys are swept twice: once for each
//            row's maximum and sum, once to rebuild, mask and apply the probabilities.
//   ANGULAR  attention with the exact angular kernel 1 - arccos(q_hat . k_hat) / pi of Eq. 4-5
//            (what the linear terms of Eq. 8 approximate), row-normalised as in Eq. 3 or not.
//
// Block = 4 waves, wave w owns queries 128 bx + 32 w .. + 31 of one unit.  Keys go through LDS in
// tiles of 32, prefetched into registers one tile ahead.  q and k enter the matrix cores as
// stored (their products are exact in fp32); the unit-row normalisation is applied to the
// products, 1 / |q_t| from a register and 1 / |k_j| from a small LDS table, so the logits carry
// no 16-bit rounding.  The probabilities are split into two 16-bit parts (value and remainder)
// for the second contraction, which keeps its error below the rounding of the output.
//   S^T[key][query] = K_tile (32 x 64) . Q^T (64 x 32): 4 x v_mfma_f32_32x32x16; lane l then
//   holds query l % 32 and the 16 keys 8 a + 4 (l / 32) + b (a, b = 0..3) of the tile;
//   out^T[ch][query] += V_tile^T (64 x 32) . P (32 x 32): the probabilities are already in
//   B-operand order (registers 8 u .. 8 u + 7 = the 8 keys of k-step u), V^T comes from the
//   [key][channel] tile through transposing LDS reads with the same key order.
#pragma once

#include "apply_mfma.hpp"
#include "common.hpp"
#include "reduce_mfma.hpp"

namespace castling {

enum { kPairSparse = 0, kPairAngular = 1 };

struct PairParams {
    int N;
    int normalize;    // SPARSE: unit rows of q and k
    int norm_none;    // ANGULAR: no division by the row sum
    int accumulate;   // add the result to what `out` holds
    float scale, threshold, eps;
    TensorStrides in, out;
};

constexpr int kPairTilePitch = 144;                 // bytes per key row of a tile
constexpr int kPairTileBytes = 32 * kPairTilePitch;

// grid = (ceil(N / 128), units), block = 256.  kept: per-unit count of entries the mask keeps
// (SPARSE; nullptr = not wanted), must be zero before the launch.
template <int MODE, typename X>
__global__ __launch_bounds__(256) void pairwise_attn_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    bf16_t* __restrict__ out, unsigned long long* __restrict__ kept, int heads, PairParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char ktile[kPairTileBytes];
    __shared__ __attribute__((aligned(16))) unsigned char vtile[kPairTileBytes];
    __shared__ __attribute__((aligned(16))) float kinv[32];  // 1 / max(|k_j|, eps) of the tile's keys

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int unit = blockIdx.y;
    const int N = p.N;
    const int hsel = lane >> 5;                 // which half of each 16-wide k-step this lane feeds
    const int qi = blockIdx.x * 128 + wave * 32 + (lane & 31);   // this lane's query
    const long long in_off = unit_offset(unit, heads, p.in);
    const bf16_t* const qb = q + in_off;
    const unsigned char* const kb = reinterpret_cast<const unsigned char*>(k + in_off);
    const unsigned char* const vb = reinterpret_cast<const unsigned char*>(v + in_off);
    const size_t in_tok = static_cast<size_t>(p.in.n) * 2;
    const float inv_eps = 1.0f / p.eps;
    const bool unit_rows = MODE == kPairAngular || p.normalize;

    // ---- this lane's query as B operands: features 16 s + 8 hsel .. + 7 for k-step s
    u32x4_t qop[4];
    float qinv;  // 1 / max(|q_t|, eps), or 1 for raw rows
    {
        const unsigned char* qrow =
            reinterpret_cast<const unsigned char*>(qb) + static_cast<size_t>(min(qi, N - 1)) * in_tok;
        float qf[32];
        float ss = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(qrow + 32 * s + 16 * hsel);
            qop[s] = raw;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                qf[8 * s + 2 * i] = X::lo(raw[i]);
                qf[8 * s + 2 * i + 1] = X::hi(raw[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) ss = fmaf(qf[i], qf[i], ss);
        ss += __shfl_xor(ss, 32, 64);  // the other half of the row
        qinv = unit_rows ? fminf(__builtin_amdgcn_rsqf(ss), inv_eps) : 1.0f;
    }

    // ---- key tiles: thread (key tid / 8, octet tid % 8) stages 16 bytes of K and of V
    const int skey = tid >> 3, soct = tid & 7;
    const int n_tiles = (N + 31) / 32;
    u32x4_t kpre, vpre;
    auto prefetch = [&](int tile, bool with_v) {
        const size_t row = static_cast<size_t>(min(32 * tile + skey, N - 1)) * in_tok + soct * 16;
        kpre = *reinterpret_cast<const u32x4_t*>(kb + row);
        if (with_v) vpre = *reinterpret_cast<const u32x4_t*>(vb + row);
    };
    auto stage = [&](int tile, bool with_v) {
        const bool in = 32 * tile + skey < N;
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        const u32x4_t kw = in ? kpre : zero;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = X::lo(kw[i]), c = X::hi(kw[i]);
            ss = fmaf(a, a, ss);
            ss = fmaf(c, c, ss);
        }
        ss = row_group_sum<8>(ss);
        if (soct == 0) kinv[skey] = unit_rows ? fminf(__builtin_amdgcn_rsqf(ss), inv_eps) : 1.0f;
        *reinterpret_cast<u32x4_t*>(ktile + skey * kPairTilePitch + soct * 16) = kw;
        if (with_v)
            *reinterpret_cast<u32x4_t*>(vtile + skey * kPairTilePitch + soct * 16) = in ? vpre : zero;
    };
    // S^T tile of this wave: register r <-> key 8 (r / 4) + 4 hsel + r % 4, this lane's query;
    // raw dot products from the matrix cores, then scaled by the two reciprocal norms and, for
    // the softmax, by scale * log2(e) (the exponentials below are base 2)
    const float qfac = MODE == kPairSparse ? qinv * p.scale * 1.44269504088896340736f : qinv;
    auto scores = [&](f32x16_t& s) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const u32x4_t a = *reinterpret_cast<const u32x4_t*>(
                ktile + (lane & 31) * kPairTilePitch + (16 * st + 8 * hsel) * 2);
            s = X::mfma32(a, qop[st], s);
        }
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            const float4 ki = *reinterpret_cast<const float4*>(kinv + 8 * a4 + 4 * hsel);
            s[4 * a4] *= qfac * ki.x;
            s[4 * a4 + 1] *= qfac * ki.y;
            s[4 * a4 + 2] *= qfac * ki.z;
            s[4 * a4 + 3] *= qfac * ki.w;
        }
    };
    // keys past N exist only in the last tile, and only if N is not a multiple of 32
    const int ragged_tile = (N & 31) ? n_tiles - 1 : -1;
    auto key_valid = [&](int r) { return 32 * (n_tiles - 1) + 8 * (r >> 2) + 4 * hsel + (r & 3) < N; };

    float row_max = -INFINITY, row_sum = 0.f;  // of the base-2 logits
    if constexpr (MODE == kPairSparse) {
        // ---- first sweep: maximum and sum of exp of every row (online, per lane, then the
        // two lanes that share a query are merged)
        prefetch(0, false);
        for (int t = 0; t < n_tiles; ++t) {
            stage(t, false);
            __syncthreads();
            if (t + 1 < n_tiles) prefetch(t + 1, false);
            f32x16_t s;
            scores(s);
            if (t == ragged_tile) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = key_valid(r) ? s[r] : -INFINITY;
            }
            float tmax = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
            const float nmax = fmaxf(row_max, tmax);
            if (nmax > -INFINITY) {
                float acc = row_sum * __builtin_amdgcn_exp2f(row_max - nmax);
#pragma unroll
                for (int r = 0; r < 16; ++r) acc += __builtin_amdgcn_exp2f(s[r] - nmax);
                row_sum = acc;
                row_max = nmax;
            }
            __syncthreads();
        }
        const float omax = __shfl_xor(row_max, 32, 64), osum = __shfl_xor(row_sum, 32, 64);
        const float m = fmaxf(row_max, omax);
        row_sum = row_sum * __builtin_amdgcn_exp2f(row_max - m) + osum * __builtin_amdgcn_exp2f(omax - m);
        row_max = m;
    }
    // SPARSE: p = 2^(logit - off); every row has at least one key, so the sum is positive
    const float off = row_max + __builtin_amdgcn_logf(row_sum);

    // ---- main sweep
    f32x16_t acc[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
    float den = 0.f;
    unsigned int n_kept = 0;  // wave total, uniform
    const bool q_valid = qi < N;
    // transposing reads of V: the 16-lane group (lane / 16) covers channels 16 (group % 2) .. + 15
    // of its k-half; source lane s of a group reads key K0 + s / 4, channels 4 (s % 4) .. + 3
    const int vsrc = ((lane >> 2) & 3) * kPairTilePitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    prefetch(0, true);
    for (int t = 0; t < n_tiles; ++t) {
        stage(t, true);
        __syncthreads();
        if (t + 1 < n_tiles) prefetch(t + 1, true);
        f32x16_t s;
        scores(s);
        if constexpr (MODE == kPairSparse) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x = __builtin_amdgcn_exp2f(s[r] - off);
                const bool keep = x > p.threshold;
                s[r] = keep ? x : 0.f;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s[r] = 1.0f - acosf(fminf(fmaxf(s[r], -1.0f), 1.0f)) * kInvPi;
        }
        if (t == ragged_tile) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = key_valid(r) ? s[r] : 0.f;
        }
        // SPARSE: (uniform per wave) a tile in which the mask kept nothing for any of the wave's
        // queries adds nothing: the usual case once the threshold bites
        bool tile_live = true;
        if constexpr (MODE == kPairSparse) {
            bool any = false;
#pragma unroll
            for (int r = 0; r < 16; ++r) any = any || s[r] != 0.f;
            tile_live = __ballot(any) != 0ull;
        }
        if (tile_live) {
            u32x4_t pop[2], plo[2];  // probabilities and their rounding remainders, 16-bit pairs
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                if constexpr (MODE == kPairSparse) {
                    // kept entries are exactly the nonzero ones (a kept probability is > thr >= 0)
                    if (kept) {
                        n_kept += __builtin_popcountll(__ballot(q_valid && s[r] != 0.f));
                        n_kept += __builtin_popcountll(__ballot(q_valid && s[r + 1] != 0.f));
                    }
                } else {
                    den += s[r] + s[r + 1];
                }
                const uint32_t hi = X::pack(s[r], s[r + 1]);
                pop[r >> 3][(r >> 1) & 3] = hi;
                plo[r >> 3][(r >> 1) & 3] = X::pack(s[r] - X::lo(hi), s[r + 1] - X::hi(hi));
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    const unsigned char* base = vtile + (16 * u + 4 * hsel) * kPairTilePitch + 64 * mt + vsrc;
                    const uint2 lo = lds_read_tr8(base);
                    const uint2 hi = lds_read_tr8(base + 8 * kPairTilePitch);
                    const u32x4_t a = {lo.x, lo.y, hi.x, hi.y};
                    acc[mt] = X::mfma32(a, pop[u], acc[mt]);
                    acc[mt] = X::mfma32(a, plo[u], acc[mt]);
                }
        }
        __syncthreads();
    }

    // ---- epilogue: this lane holds, for its query, channels 32 mt + 8 a + 4 hsel + b
    float post = 1.0f;
    if constexpr (MODE == kPairAngular) {
        den += __shfl_xor(den, 32, 64);
        if (!p.norm_none) post = 1.0f / den;
    }
    if (qi < N) {
        unsigned char* orow = reinterpret_cast<unsigned char*>(out + unit_offset(unit, heads, p.out)) +
                              static_cast<size_t>(qi) * (static_cast<size_t>(p.out.n) * 2);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                uint2* dst = reinterpret_cast<uint2*>(orow + (32 * mt + 8 * a + 4 * hsel) * 2);
                float r0 = acc[mt][4 * a] * post, r1 = acc[mt][4 * a + 1] * post;
                float r2 = acc[mt][4 * a + 2] * post, r3 = acc[mt][4 * a + 3] * post;
                if (p.accumulate) {
                    const uint2 old = *dst;
                    r0 += X::lo(old.x);
                    r1 += X::hi(old.x);
                    r2 += X::lo(old.y);
                    r3 += X::hi(old.y);
                }
                uint2 o;
                o.x = X::pack(r0, r1);
                o.y = X::pack(r2, r3);
                *dst = o;
            }
    }
    if constexpr (MODE == kPairSparse) {
        if (kept && lane == 0) atomicAdd(kept + unit, static_cast<unsigned long long>(n_kept));
    }
}

// grid = (ceil(n / 256)), block = 256
__global__ __launch_bounds__(256) void zero_u64_kernel(unsigned long long* p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

}  // namespace castling
