// Pass 2 for bf16 / fp16 I/O on the matrix cores: heads of 64 channels, or two neighbouring
// heads of 32 channels as one unit (PAIR).
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
// Work unit: a strip of 16 grid columns of one (batch, head) unit, four output rows per
// stage, walked top to bottom by a persistent block (one per compute unit).
// A block has twelve waves, three per SIMD, one of each role:
//   waves 0..3   consumers: wave c owns channels 16c..16c+15; it keeps a ring of DWConv data
//                operands (12 grid rows for a 9x9 filter) in registers, runs the 4x4x4 MFMAs
//                for the four output rows of the stage with the linear branch as the C
//                operand, and writes its results to an LDS output tile;
//   waves 4..7   stagers: asynchronous V loads (several stages ahead), transposition of the V
//                rows into the MFMA operand order (transposing LDS reads), and the coalesced
//                stores of finished output tiles;
//   waves 8..11  linear: asynchronous Q loads and the linear branch of row p of the stage,
//                software-pipelined over two stages (matrix products of the next stage are
//                issued before the current one is finished).
// Stagers and linear waves work one stage ahead of the consumers; all meet at one LDS-only
// barrier per stage.
#pragma once

#include <type_traits>
#include <utility>

#include "common.hpp"
#include "reduce_mfma.hpp"

namespace castling {


struct ApplyMfmaParams {
    int N, grid_h, grid_w;
    int strips;     // 16-column strips per grid row
    int norm_none, do_linear, do_dwconv;
    float eps;
    TensorStrides in, out;  // of q and v; of out.  N * token stride * 2 stays below 4 GiB
    // Pairs of 32-wide heads run as one 64-channel unit: bytes to add to the address of the
    // second half of a token row (channels 32..63 belong to the next head); 0 otherwise
    uint32_t in_skew, out_skew;
    float lin_scale;  // factor on the linear branch where there is no normaliser (1 in the forward)
};

constexpr int kStripW = 16;
// V operand tile of one stage: [row 4][quad 6][channel 64] units of 8 bytes (4 consecutive
// tokens of one channel); octets of channels are 80 bytes apart, quads 672 (bank spread)
constexpr int kVtQuadStride = 672;
constexpr int kVtOctetStride = 80;
constexpr int kVtRowStride = 6 * kVtQuadStride;
constexpr int kVtBytes = 4 * kVtRowStride;
constexpr int kVtBuffers = 2;
// linear-branch tile of one stage: [row 4][channel 64][token 16 + pad] fp32
constexpr int kLinTokPitch = 20;
constexpr int kLinBytes = 4 * 64 * kLinTokPitch * 4;
// output tile of one stage: [row 4][channel 64][token 16 + pad] bf16
constexpr int kOutTokPitch = 20;
constexpr int kOutBytes = 4 * 64 * kOutTokPitch * 2;
// per stager wave and V item: 8 tokens x 64 channels in global (token-major) order
constexpr int kNatTokPitch = 144;
constexpr int kNatBytes = 3 * 8 * kNatTokPitch;
// per stager wave: one finished output row of the strip, 16 tokens x 64 channels token-major
constexpr int kRowBytes = 16 * kNatTokPitch;
constexpr int kApplyWaves = 12;
constexpr int kApplyMfmaLdsBytes =
    kVtBuffers * kVtBytes + 2 * kLinBytes + 2 * kOutBytes + 4 * kNatBytes + 4 * kRowBytes;

// ---------------------------------------------------------------------------
// Work is cut into "steps" of 4 output rows of one 16-column strip of one unit.
// Steps are numbered unit-major, then strip, then top to bottom; logical block b of G
// takes the contiguous range [b*T/G, (b+1)*T/G) of the T steps, so every compute
// unit gets the same amount of work whatever the grid shape.  Workgroups are handed to
// the 8 XCDs in turn, so workgroup i is logical block (i % 8) * (G / 8) + i / 8: the
// blocks of one XCD then cover neighbouring strips, whose halo columns meet in its L2.  A maximal run of
// steps inside one strip column is a segment; a segment first primes the DWConv
// window (NCH - 1 stages that only stage V rows) and then emits one step per stage.
// After the last stage the cursor stays where it is with live = false: the prefetches
// issued past the end repeat the last stage's loads and are never consumed.
struct StageCursor {
    int g_begin, g_end;  // steps [g_begin, g_end) of the current segment
    int t;               // stage inside the segment
    int range_end;       // end of this block's step range
    int unit, strip;     // strip column of the segment
    int y0;              // first output row of the segment
    bool live;

    // divisions happen here only; the loop advances with adds and compares
    __device__ __forceinline__ void start(int s0, int s1, int spc, int strips)
    {
        range_end = s1;
        g_begin = s0;
        const int col = s0 / spc;
        g_end = min(s1, (col + 1) * spc);
        unit = col / strips;
        strip = col - unit * strips;
        y0 = 4 * (s0 - col * spc);
        t = 0;
        live = s0 < s1;
    }
    __device__ __forceinline__ void advance(int spc, int strips, int nch)
    {
        if (!live) return;
        if (++t == (g_end - g_begin) + nch - 1) {  // next segment starts a new strip column
            if (g_end >= range_end) {
                live = false;
                --t;
                return;
            }
            g_begin = g_end;
            g_end = min(range_end, g_begin + spc);
            y0 = 0;
            t = 0;
            if (++strip == strips) {
                strip = 0;
                ++unit;
            }
        }
    }
    // first output row of the stage (valid when computes(nch))
    __device__ __forceinline__ int yo(int nch) const { return y0 + 4 * (t - (nch - 1)); }
    __device__ __forceinline__ bool computes(int nch) const { return live && t >= nch - 1; }
};

// LDS-only workgroup barrier: global loads that are still in flight stay in flight.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// 16-byte store of output that is not read again by this layer (non-temporal)
__device__ __forceinline__ void store16_stream(void* p, uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t v4;
    const v4 val = {a, b, c, d};
    __builtin_nontemporal_store(val, reinterpret_cast<v4*>(p));
}

// 8-byte transposing LDS read (see lds_operand_tr in reduce_mfma.hpp for the lane roles)
__device__ __forceinline__ uint2 lds_read_tr8(const unsigned char* addr)
{
    typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(addr));
    return __builtin_bit_cast(uint2, r);
}

constexpr int kApplyPrefetch = 2;   // stages whose global loads are in flight
constexpr int kLinearPrefetch = 4;  // the same for the linear waves' q

// what a wave needs to know about a stage after its cursor has moved on
struct StageSnap {
    int unit, xs0, yo;
    bool computes;
    long long obase;  // element offset of the unit in out (stagers only)
};

// grid = (G), block = 64 * kApplyWaves.
// PAIR: a unit is two heads of 32 channels.  Loads, stores and the convolution do not care; the
// linear branch takes each half's norm, row sum and state from its own head (the S operand
// table is then block diagonal, and only the matching half of q meets it).
template <int KS, bool LIN, bool DW, typename X, bool PAIR = false>
__global__ __launch_bounds__(64 * kApplyWaves) void apply_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ v, const bf16_t* __restrict__ bias,
    const bf16_t* __restrict__ sfrag, const bf16_t* __restrict__ kfrag,
    const float* __restrict__ vhalf, const bf16_t* __restrict__ wfrag, bf16_t* __restrict__ out,
    int heads, int total_steps, ApplyMfmaParams p)
{
    constexpr int D = 64;
    constexpr int RAD = KS / 2;
    constexpr int NCH = (KS + 3 + 3) / 4;  // stages until a segment's first output
    constexpr int WR = 4 * NCH;            // rows in a consumer's operand ring
    constexpr int PD = kApplyPrefetch;
    static_assert(PD % 2 == 0, "the two-deep LDS rings assume an even prefetch depth");

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave >> 2;   // 0 consumer, 1 stager, 2 linear
    const int c = wave & 3;       // channel group / stager index / row inside the stage
    const int W = p.grid_w, H = p.grid_h;
    const int spc = (H + 3) / 4;  // steps per strip column
    const uint32_t in_tok = static_cast<uint32_t>(p.in.n) * 2;    // bytes between tokens
    const uint32_t out_tok = static_cast<uint32_t>(p.out.n) * 2;

    // consecutive workgroups go to the 8 XCDs in turn: give each XCD a contiguous step range
    const int lblock = (gridDim.x % 8 == 0) ? (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8
                                            : static_cast<int>(blockIdx.x);
    const int s_begin = static_cast<int>(static_cast<long long>(lblock) * total_steps / gridDim.x);
    const int s_end = static_cast<int>(static_cast<long long>(lblock + 1) * total_steps / gridDim.x);

    unsigned char* const vt_base = lds;
    unsigned char* const lin_base = lds + kVtBuffers * kVtBytes;
    unsigned char* const out_base = lin_base + 2 * kLinBytes;
    unsigned char* const nat_base = out_base + 2 * kOutBytes;

    // stages of this block
    int n_stages = 0;
    {
        StageCursor cu;
        cu.start(s_begin, s_end, spc, p.strips);
        int gb = cu.g_begin, ge = cu.g_end;
        while (gb < s_end) {
            n_stages += (ge - gb) + NCH - 1;
            gb = ge;
            ge = min(s_end, gb + spc);
        }
    }
    if (n_stages == 0) return;  // uniform per block; the host never launches such a block

    // The stager and linear waves have little work per stage, but the consumers' MFMA
    // stream would starve them of issue slots; they run at a raised wave priority.
    if (role != 0) __builtin_amdgcn_s_setprio(2);

    if (role == 1) {
        // ======================================================== stager waves
        constexpr int YOUNGER = (PD - 1) * 3;  // loads issued after a stage's own
        const int stid = tid & 255;            // index among the 256 stager threads
        const int tl = lane & 15;
        u32x4_t vreg[PD][3];
        uint32_t okmask[PD];  // bit it: V item it lies inside the grid
        StageSnap snap[PD];   // stage held by each register slot
        StageSnap fsnap[2];   // stages whose output tiles wait to be stored
        fsnap[0].computes = fsnap[1].computes = false;
        fsnap[0].unit = fsnap[1].unit = 0;
        fsnap[0].xs0 = fsnap[1].xs0 = fsnap[0].yo = fsnap[1].yo = 0;
        fsnap[0].obase = fsnap[1].obase = 0;
        int base_unit = -1;  // unit whose offsets are cached (uniform per block)
        long long v_base = 0, o_base = 0;

        // this thread's three V items (of 4 rows x 24 columns x 8 octets): a wave covers,
        // per item, 8 consecutive columns (two quads) of one row with all 64 channels
        int v_r[3], v_x[3];
#pragma unroll
        for (int it = 0; it < 3; ++it) {
            const int item = stid + 256 * it;
            v_r[it] = item / 192;
            v_x[it] = ((item % 192) >> 3) - 4;
        }
        const int v_oct = lane & 7;
        const uint32_t v_oct_off = v_oct * 16 + (v_oct >> 2) * p.in_skew;
        const uint32_t o_oct_off = v_oct * 16 + (v_oct >> 2) * p.out_skew;
        unsigned char* const nat = nat_base + c * kNatBytes;
        // transposition roles: token-major write (token lane/8, octet lane%8); transposing read
        // source (token 4 qd + (lane/4)%4, channels 16 (lane/16) + 4 (lane%4)..+3); afterwards
        // lane l holds channel l, 4 tokens of quad qd
        unsigned char* const nat_wr = nat + (lane >> 3) * kNatTokPitch + v_oct * 16;
        const unsigned char* const nat_rd =
            nat + ((lane >> 2) & 3) * kNatTokPitch + (16 * (lane >> 4) + 4 * (lane & 3)) * 2;
        const int vt_lane = (lane >> 3) * kVtOctetStride + (lane & 7) * 8;
        // output tile: stager c stores row c of the stage.  A transposing read gives lane l token
        // l % 16 and octet l / 16 (+ 4 in the second pass); the row then goes through a
        // wave-private token-major copy so that each store instruction writes 8 whole 128-byte
        // lines (lane l: token l / 8 (+ 8), octet l % 8).  Half-line non-temporal stores cost
        // extra memory writes.
        const int fl_off = (((lane >> 2) & 3) * kOutTokPitch + 4 * (lane & 3)) * 2;
        unsigned char* const orow = nat_base + 4 * kNatBytes + c * kRowBytes;
        unsigned char* const orow_wr = orow + tl * kNatTokPitch + (lane >> 4) * 16;
        const unsigned char* const orow_rd = orow + (lane >> 3) * kNatTokPitch + (lane & 7) * 16;

        auto issue_loads = [&](auto slot_c, const StageCursor& cu) {
            constexpr int slot = decltype(slot_c)::value;
            const int xs0 = cu.strip * kStripW;
            if (cu.unit != base_unit) {
                base_unit = cu.unit;
                v_base = unit_offset(cu.unit, heads, p.in);
                o_base = unit_offset(cu.unit, heads, p.out);
            }
            const bf16_t* vb = v + v_base;
            const int row_base = cu.y0 - RAD + 4 * cu.t;
            uint32_t ok = 0;
            if constexpr (DW) {
#pragma unroll
                for (int it = 0; it < 3; ++it) {
                    const int gy = row_base + v_r[it], gx = xs0 + v_x[it];
                    if (gy >= 0 && gy < H && gx >= 0 && gx < W) ok |= 1u << it;
                    const int cy = min(max(gy, 0), H - 1), cx = min(max(gx, 0), W - 1);
                    async_load16(vreg[slot][it], vb,
                                 static_cast<uint32_t>(cy * W + cx) * in_tok + v_oct_off);
                }
            }
            okmask[slot] = ok;
            snap[slot].obase = o_base;
            snap[slot].unit = cu.unit;
            snap[slot].xs0 = xs0;
            snap[slot].yo = cu.yo(NCH);
            snap[slot].computes = cu.computes(NCH);
        };

        // row c of output tile `ot` -> this lane's 16 bytes of two groups of 8 whole token rows
        auto load_out_row = [&](const unsigned char* ot, u32x4_t (&line)[2]) {
            uint2 f_lo[2], f_hi[2];
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int oct = (lane >> 4) + 4 * it;
                const unsigned char* src = ot + (c * 64 + 8 * oct) * (kOutTokPitch * 2) + fl_off;
                f_lo[it] = lds_read_tr8(src);
                f_hi[it] = lds_read_tr8(src + 4 * kOutTokPitch * 2);
            }
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const u32x4_t val = {f_lo[it].x, f_lo[it].y, f_hi[it].x, f_hi[it].y};
                *reinterpret_cast<u32x4_t*>(orow_wr + it * 64) = val;
            }
            __builtin_amdgcn_wave_barrier();  // wave-private: LDS operations complete in issue order
#pragma unroll
            for (int it = 0; it < 2; ++it)
                line[it] = *reinterpret_cast<const u32x4_t*>(orow_rd + it * 8 * kNatTokPitch);
            __builtin_amdgcn_wave_barrier();
        };
        auto store_out_row = [&](unsigned char* ou, const StageSnap& fs, const u32x4_t (&line)[2]) {
            const int y = fs.yo + c;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int x = fs.xs0 + (lane >> 3) + 8 * it;
                if (y < H && x < W)
                    store16_stream(ou + (static_cast<uint32_t>(y * W + x) * out_tok + o_oct_off),
                                   line[it][0], line[it][1], line[it][2], line[it][3]);
            }
        };

        auto stage_v = [&](auto slot_c, const StageSnap& fs, const unsigned char* ot, unsigned char* vt) {
            constexpr int slot = decltype(slot_c)::value;
            // finished output tile: fetched and re-laid now, stored once the V work is issued
            u32x4_t line[2];
            load_out_row(ot, line);
            if constexpr (DW) {
                const uint32_t ok = okmask[slot];
                wait_async_loads<YOUNGER>(vreg[slot][0], vreg[slot][1], vreg[slot][2]);
                // token-major staging, private to this wave; LDS operations of one wave
                // complete in issue order, so no barrier is needed around it
#pragma unroll
                for (int it = 0; it < 3; ++it) {
                    const u32x4_t zero = {0u, 0u, 0u, 0u};
                    *reinterpret_cast<u32x4_t*>(nat_wr + it * 8 * kNatTokPitch) =
                        ((ok >> it) & 1u) ? vreg[slot][it] : zero;
                }
                __builtin_amdgcn_wave_barrier();
            }
            if (fs.computes) {
                unsigned char* ou = reinterpret_cast<unsigned char*>(out + fs.obase);
                store_out_row(ou, fs, line);
            }
            if constexpr (DW) {
                uint2 u[3][2];
#pragma unroll
                for (int it = 0; it < 3; ++it)
#pragma unroll
                    for (int qd = 0; qd < 2; ++qd)
                        u[it][qd] = lds_read_tr8(nat_rd + (it * 8 + qd * 4) * kNatTokPitch);
#pragma unroll
                for (int it = 0; it < 3; ++it) {
                    const int item0 = c * 64 + 256 * it;  // first item of this wave
                    const int r = item0 / 192, x0 = (item0 % 192) >> 3;
                    unsigned char* dst = vt + (r * 6 + (x0 >> 2)) * kVtQuadStride + vt_lane;
#pragma unroll
                    for (int qd = 0; qd < 2; ++qd)
                        *reinterpret_cast<uint2*>(dst + qd * kVtQuadStride) = u[it][qd];
                }
                __builtin_amdgcn_wave_barrier();
            }
        };

        StageCursor ld;
        ld.start(s_begin, s_end, spc, p.strips);
        static_for<PD>([&](auto slot) {
            issue_loads(slot, ld);
            ld.advance(spc, p.strips, NCH);
        });
        for (int s = 0; s < n_stages; s += PD) {
            static_for<PD>([&](auto slot) {
                if (s + decltype(slot)::value >= n_stages) return;
                constexpr int b2 = decltype(slot)::value & 1;
                // the output tile two stages back is complete
                stage_v(slot, fsnap[b2], out_base + b2 * kOutBytes, vt_base + b2 * kVtBytes);
                fsnap[b2] = snap[decltype(slot)::value];
                // refill the slot that was just drained (past the end the cursor stands still and
                // the loads repeat the last stage's: the count of loads in flight stays fixed)
                issue_loads(slot, ld);
                ld.advance(spc, p.strips, NCH);
                lds_barrier();
            });
        }
        // the last two tiles: a pass with nothing to stage but the stores
        auto flush_only = [&](const StageSnap& fs, const unsigned char* ot) {
            if (!fs.computes) return;
            unsigned char* ou = reinterpret_cast<unsigned char*>(out + fs.obase);
            u32x4_t line[2];
            load_out_row(ot, line);
            store_out_row(ou, fs, line);
        };
        // stage n - 2 (tile parity n % 2) is complete; stage n - 1 is after one more barrier
        if (n_stages & 1) {
            flush_only(fsnap[1], out_base + kOutBytes);
            lds_barrier();
            flush_only(fsnap[0], out_base);
        } else {
            flush_only(fsnap[0], out_base);
            lds_barrier();
            flush_only(fsnap[1], out_base + kOutBytes);
        }
        // drain the loads issued past the end before the registers die
        if constexpr (DW)
            static_for<PD>([&](auto slot) {
                wait_async_loads<0>(vreg[slot][0], vreg[slot][1], vreg[slot][2]);
            });
    } else if (role == 2) {
        // ======================================================== linear waves
        // Software pipeline over two stages: in the interval of stage s the wave first issues
        // the matrix products of stage s + 1 (phase A: wait for its q, MFMAs into the other
        // accumulator set) and then finishes stage s (phase B: norms, reciprocals, the linear
        // tile) while those products run.  Its loads are LPD stages ahead.
        constexpr int LPD = kLinearPrefetch;
        static_assert(LPD % 2 == 0, "tile parity is taken from the slot index");
        constexpr int YOUNGER = (LPD - 1) * 2;
        const int tl = lane & 15, g = lane >> 4;
        const float inv_eps = 1.0f / p.eps, half_n = 0.5f * static_cast<float>(p.N);
        u32x4_t sf[4][2], kf[2];
        const float unsc = X::table_unscale(p.N);
        float vh[4] = {0.f, 0.f, 0.f, 0.f};
        int lin_unit = -1;
        u32x4_t qreg[LPD][2];
        bool qok[LPD];
        StageSnap snap[LPD];
        int base_unit = -1;
        long long q_base = 0;
        // products of two stages in flight: [parity]
        f32x4_t gram[2], dk[2], acc[2][4];
        f32x4_t gramb[2], dkb[2];  // PAIR: the same for the second head of the pair
        float vhb[2][4];
        bool busy[2] = {false, false};

        auto issue_loads = [&](auto slot_c, const StageCursor& cu) {
            constexpr int slot = decltype(slot_c)::value;
            const int xs0 = cu.strip * kStripW;
            if constexpr (LIN) {
                const int y = cu.yo(NCH) + c, x = xs0 + tl;
                qok[slot] = cu.computes(NCH) && y < H && x < W;
                const int cy = min(max(y, 0), H - 1), cx = min(x, W - 1);
                const uint32_t off = static_cast<uint32_t>(cy * W + cx) * in_tok + g * 16;
                if (cu.unit != base_unit) {
                    base_unit = cu.unit;
                    q_base = unit_offset(cu.unit, heads, p.in);
                }
                const bf16_t* qb = q + q_base;
                async_load16_stream(qreg[slot][0], qb, off);
                async_load16_stream(qreg[slot][1], qb, off + 64 + p.in_skew);
            }
            snap[slot].unit = cu.unit;
            snap[slot].xs0 = xs0;
            snap[slot].yo = cu.yo(NCH);
            snap[slot].computes = cu.computes(NCH);
        };

        // phase A of the stage held in `slot`, into accumulator set PAR
        auto products = [&](auto slot_c, auto par_c) {
            constexpr int slot = decltype(slot_c)::value;
            constexpr int PAR = decltype(par_c)::value;
            if constexpr (LIN) {
                wait_async_loads<YOUNGER>(qreg[slot][0], qreg[slot][1]);
                busy[PAR] = snap[slot].computes;
                if (!snap[slot].computes) return;
                const int unit = snap[slot].unit;
                if (unit != lin_unit) {  // uniform per block: operand tables of the new unit
                    lin_unit = unit;
                    const uint4* s4 = reinterpret_cast<const uint4*>(
                        sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
                    const uint4* k4 = reinterpret_cast<const uint4*>(
                        kfrag + static_cast<size_t>(unit) * kKfragPerUnit);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks)
                            sf[nt][ks] = __builtin_bit_cast(u32x4_t, s4[(nt * 2 + ks) * 64 + lane]);
                        vh[nt] = vhalf[unit * D + 16 * nt + tl];
                    }
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
                        kf[ks] = __builtin_bit_cast(u32x4_t, k4[ks * 64 + lane]);
                }
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) vhb[PAR][nt] = vh[nt];
                const u32x4_t zero = {0u, 0u, 0u, 0u};
                u32x4_t a[2];
                a[0] = qok[slot] ? qreg[slot][0] : zero;
                a[1] = qok[slot] ? qreg[slot][1] : zero;
                // |q_t|^2 on the matrix cores: the diagonal of Q Q^T (B operand = same registers).
                // Six independent accumulators, k-step outermost: no MFMA waits for the one
                // issued just before it.
                if constexpr (PAIR) {
                    // k-step 0 holds the first head's 32 features, k-step 1 the second's
                    const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
                    gram[PAR] = X::mfma16(a[0], a[0], z);
                    gramb[PAR] = X::mfma16(a[1], a[1], z);
                    dk[PAR] = X::mfma16(a[0], kf[0], z);
                    dkb[PAR] = X::mfma16(a[1], kf[1], z);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
                        acc[PAR][nt] = X::mfma16(a[nt >> 1], sf[nt][nt >> 1], z);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) gram[PAR][r] = dk[PAR][r] = 0.f;
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[PAR][nt][r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        gram[PAR] = X::mfma16(a[ks], a[ks], gram[PAR]);
                        dk[PAR] = X::mfma16(a[ks], kf[ks], dk[PAR]);
#pragma unroll
                        for (int nt = 0; nt < 4; ++nt)
                            acc[PAR][nt] = X::mfma16(a[ks], sf[nt][ks], acc[PAR][nt]);
                    }
                }
            }
        };

        // phase B of the stage whose products sit in accumulator set PAR
        auto finish = [&](auto par_c, float* lin) {
            constexpr int PAR = decltype(par_c)::value;
            if constexpr (LIN) {
                if (!busy[PAR]) return;
                constexpr int NH = PAIR ? 2 : 1;  // heads in the unit
                float alpha[NH][4], beta[NH][4];
#pragma unroll
                for (int hh = 0; hh < NH; ++hh)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float gr = hh ? gramb[PAR][r] : gram[PAR][r];
                        const float dr = hh ? dkb[PAR][r] : dk[PAR][r];
                        // entry (m, m) of the Gram tile, m = 4 g + r, sits in lane 16 (m / 4) + m, register m % 4
                        const float ssr = __int_as_float(
                            __builtin_amdgcn_ds_bpermute((20 * g + r) * 4, __float_as_int(gr)));
                        // 1 / max(|q|, eps) with the hardware reciprocal square root (1 ulp)
                        float inv = fminf(__builtin_amdgcn_rsqf(ssr), inv_eps);
                        if constexpr (X::kHalf) inv *= unsc;  // the tables are scaled down
                        if (p.norm_none) {
                            alpha[hh][r] = inv * p.lin_scale;
                            beta[hh][r] = p.lin_scale;
                        } else {
                            const float rden = __builtin_amdgcn_rcpf(half_n + inv * dr);
                            alpha[hh][r] = inv * rden;
                            beta[hh][r] = rden;
                        }
                    }
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const int hh = PAIR ? (nt >> 1) : 0;
                    float4 o;
                    o.x = fmaf(alpha[hh][0], acc[PAR][nt][0], beta[hh][0] * vhb[PAR][nt]);
                    o.y = fmaf(alpha[hh][1], acc[PAR][nt][1], beta[hh][1] * vhb[PAR][nt]);
                    o.z = fmaf(alpha[hh][2], acc[PAR][nt][2], beta[hh][2] * vhb[PAR][nt]);
                    o.w = fmaf(alpha[hh][3], acc[PAR][nt][3], beta[hh][3] * vhb[PAR][nt]);
                    *reinterpret_cast<float4*>(lin + ((c * 64 + 16 * nt + tl) * kLinTokPitch + 4 * g)) = o;
                }
            }
        };

        StageCursor ld;
        ld.start(s_begin, s_end, spc, p.strips);
        static_for<LPD>([&](auto slot) {
            issue_loads(slot, ld);
            ld.advance(spc, p.strips, NCH);
        });
        // stage 0: its products, then the refill of its slot
        products(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        issue_loads(std::integral_constant<int, 0>{}, ld);
        ld.advance(spc, p.strips, NCH);
        for (int s = 0; s < n_stages; s += LPD) {
            static_for<LPD>([&](auto i_c) {
                constexpr int i = decltype(i_c)::value;          // stage s + i, slot i, parity i % 2
                if (s + i >= n_stages) return;
                constexpr int next = (i + 1) % LPD;
                if (s + i + 1 < n_stages) {
                    products(std::integral_constant<int, next>{}, std::integral_constant<int, next & 1>{});
                    // refill the slot just read (past the end the cursor stands still and the
                    // loads repeat the last stage's: the count of loads in flight stays fixed)
                    issue_loads(std::integral_constant<int, next>{}, ld);
                    ld.advance(spc, p.strips, NCH);
                }
                finish(std::integral_constant<int, i & 1>{},
                       reinterpret_cast<float*>(lin_base + (i & 1) * kLinBytes));
                lds_barrier();
            });
        }
        lds_barrier();
        if constexpr (LIN)
            static_for<LPD>([&](auto slot) { wait_async_loads<0>(qreg[slot][0], qreg[slot][1]); });
    } else {
        // ======================================================== consumer waves
        const int blk = lane >> 2, j = lane & 3;
        const int ch_dw = 16 * c + blk;
        s16x4_t tw[KS][3];
        s16x4_t win[WR][3];  // ring: stage s writes rows 4 (s % NCH) .. +3
        float bias_dw = 0.f;
        int cons_unit = -1;
#pragma unroll
        for (int a = 0; a < WR; ++a)
#pragma unroll
            for (int m = 0; m < 3; ++m) win[a][m] = s16x4_t{0, 0, 0, 0};
#pragma unroll
        for (int a = 0; a < KS; ++a)
#pragma unroll
            for (int m = 0; m < 3; ++m) tw[a][m] = s16x4_t{0, 0, 0, 0};
        const int vt_lane = (ch_dw >> 3) * kVtOctetStride + (ch_dw & 7) * 8 + j * kVtQuadStride;

        auto consume = [&](auto ph_c, const StageCursor& cu, const unsigned char* vt, const float* lin,
                           unsigned char* ot) {
            constexpr int ph = decltype(ph_c)::value;  // stage index modulo NCH: ring phase
            if constexpr (DW) {
                if (cu.unit != cons_unit) {  // uniform per block: Toeplitz operands of the unit's head
                    cons_unit = cu.unit;
                    const int head = cu.unit % heads;
                    const uint2* wf = reinterpret_cast<const uint2*>(wfrag) +
                                      ((static_cast<size_t>(head) * 4 + c) * KS * 3) * 64 + lane;
#pragma unroll
                    for (int dy = 0; dy < KS; ++dy)
#pragma unroll
                        for (int m = 0; m < 3; ++m)
                            tw[dy][m] = __builtin_bit_cast(s16x4_t, wf[(dy * 3 + m) * 64]);
                    bias_dw = bias ? X::one(bias[head * D + ch_dw]) : 0.f;
                }
                // the four staged rows replace the oldest four of the ring
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int m = 0; m < 3; ++m)
                        win[4 * ph + r][m] = __builtin_bit_cast(
                            s16x4_t,
                            *reinterpret_cast<const uint2*>(vt + r * kVtRowStride + m * kVtQuadStride + vt_lane));
            }
            if (!cu.computes(NCH)) return;

            f32x4_t acc[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                if constexpr (LIN) {
                    const float4 l4 = *reinterpret_cast<const float4*>(
                        lin + ((rr * 64 + ch_dw) * kLinTokPitch + 4 * j));
                    acc[rr][0] = l4.x + bias_dw;
                    acc[rr][1] = l4.y + bias_dw;
                    acc[rr][2] = l4.z + bias_dw;
                    acc[rr][3] = l4.w + bias_dw;
                } else {
                    acc[rr][0] = acc[rr][1] = acc[rr][2] = acc[rr][3] = bias_dw;
                }
            }
            if constexpr (DW) {
                // input row (yo - RAD + i) is ring row (4 (ph + 1) + i) mod WR
#pragma unroll
                for (int dy = 0; dy < KS; ++dy)
#pragma unroll
                    for (int m = 0; m < 3; ++m)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            acc[rr] = X::mfma4(tw[dy][m], win[(4 * (ph + 1) + rr + dy) % WR][m], acc[rr]);
            }
            // results go to the LDS output tile [row][channel][token]
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                uint2 o;
                o.x = X::pack(acc[rr][0], acc[rr][1]);
                o.y = X::pack(acc[rr][2], acc[rr][3]);
                *reinterpret_cast<uint2*>(ot + ((rr * 64 + ch_dw) * kOutTokPitch + 4 * j) * 2) = o;
            }
        };

        StageCursor cs;
        cs.start(s_begin, s_end, spc, p.strips);
        lds_barrier();
        for (int s = 0; s < n_stages; s += NCH) {
            static_for<NCH>([&](auto ph) {
                if (s + decltype(ph)::value < n_stages) {
                    const int b2 = (s + decltype(ph)::value) & 1;
                    consume(ph, cs, vt_base + b2 * kVtBytes,
                            reinterpret_cast<const float*>(lin_base + b2 * kLinBytes),
                            out_base + b2 * kOutBytes);
                    cs.advance(spc, p.strips, NCH);
                    lds_barrier();
                }
            });
        }
    }
}

}  // namespace castling
