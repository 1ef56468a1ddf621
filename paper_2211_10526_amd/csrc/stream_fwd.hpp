// The whole layer in one launch for bf16 / fp16 heads of 64 channels: pass 1 (K normalisation and
// the token reduction of Sec. 3.1), the ordered sum of its partial states, and pass 2 (Q
// normalisation, Eq. 3 with the linear terms of Eq. 8, the DWConv term of Eq. 9) run as tasks
// of one persistent kernel.
//
// Why one launch: the state of a unit needs all of its tokens before any output row, so V is
// read twice.  A unit's tasks are all served by the workgroups of one XCD (workgroups are dealt
// to the eight XCDs in turn, so workgroup i runs on XCD i % 8): pass 2 of a unit starts as soon
// as its state is complete and finds V in that XCD's L2.  K, Q and the output go through the
// L2 with non-temporal hints, which leaves the lines of V in place.
//
// Scheduling: the host writes one task list per XCD in an order in which every task comes after
// the tasks it waits for (reduce chunks of a unit, then its combine slices, then its apply
// chunks, with the reduce chunks of the next unit dealt in between).  A workgroup claims the
// next task of its XCD's list with an atomic ticket and, where the task depends on others,
// polls their completion counter.  A task is only claimed after all earlier ones of the list
// have been claimed by workgroups that are running, so every wait ends (the poll still gives up
// after `spin_limit` rounds and sets the error word).  The last workgroup to leave resets the
// counters: a forward needs no memset and can be captured in a graph.
//
// What crosses workgroups inside the launch (partial states, operand tables, counters) is
// written and read with device-scope accesses (see st_agent); the producer waits for its stores
// (s_waitcnt vmcnt(0), then the workgroup barrier) before it bumps the counter.
//
// Pass 2 of a workgroup (4 waves, two workgroups per compute unit): a strip of 16 grid columns,
// 4 output rows per stage.  Every wave does a quarter of each job of a stage:
//   loads    V rows of the stage after next (4 rows x 24 columns, 16 + halo) and the q rows,
//            16-byte global loads whose landing the wave tracks itself;
//   staging  V: token-major into a wave-private LDS tile, read back with the transposing LDS read
//            (lane = channel, 4 consecutive tokens) and written to the operand tile
//            [row][quad][channel]; q: 1/|q| and the row sum of Eq. 3 on the vector ALU
//            (two-element dot products on the raw pairs), q rows and the two per-token factors
//            to LDS;
//   products wave c owns channels 16c..16c+15: q . S/pi for its 16 output channels on the
//            16x16x32 MFMA, moved to the lanes of the convolution with four lane permutes
//            and used as its C operand; the depthwise k x k filter as a banded Toeplitz
//            product along x on the 16-block 4x4x4 MFMA (one block per channel), the last
//            4 * NCH input rows kept in registers;
//   stores   wave r writes output row r of the previous stage: transposing read of the
//            [channel][token] tile, a wave-private token-major copy, whole 128-byte lines.
// One LDS-only barrier per stage.
#pragma once

#include "common.hpp"
#include "formats.hpp"
#include "reduce_mfma.hpp"
#include "tables.hpp"

namespace castling {

// ---------------------------------------------------------------- tasks and counters
enum : uint32_t { kTaskWeights = 0, kTaskReduce = 1, kTaskCombine = 2, kTaskApply = 3 };
constexpr uint32_t kTaskNone = 0xffffffffu;
constexpr int kTaskMaxChunks = 4096, kTaskMaxUnits = 65536;
__host__ __device__ constexpr uint32_t make_task(uint32_t kind, uint32_t unit, uint32_t chunk)
{
    return (kind << 28) | (unit << 12) | chunk;
}

// words of the counter block
constexpr int kCtrHead = 0;        // + 32 * queue: next ticket of the queue
constexpr int kCtrDone = 8 * 32;   // workgroups that have left
constexpr int kCtrWeights = 9 * 32;   // weight tasks done
constexpr int kCtrError = 10 * 32;    // sticky: first word = code of the first problem (0 = none), then details
constexpr int kCtrUnit = 11 * 32;  // + 2 * unit: reduce chunks done; + 1: state ready (slices done)
constexpr int kStreamQueues = 8;
__host__ __device__ constexpr size_t stream_counter_words(int units) { return kCtrUnit + 2 * static_cast<size_t>(units); }

// codes of the error word
enum : uint32_t {
    kStreamErrWait = 1,     // a poll for other tasks' results gave up
    kStreamErrTask = 2,     // a task word outside the launch's ranges
    kStreamErrLoad = 3,     // pass 2: a load offset outside the unit
    kStreamErrStore = 4,    // pass 2: a store offset outside the unit
};

constexpr int kWeightEntriesPerTask = 2048;   // 8-byte entries of the filter operand table
constexpr int kCombineEntries = 2048 + 128 + 32;  // S pairs, column sums, ksum pairs

struct StreamArgs {
    const bf16_t* q;
    const bf16_t* k;
    const bf16_t* v;
    const bf16_t* w;      // filters to convert in this launch, or nullptr: wfrag is ready
    const bf16_t* bias;
    bf16_t* out;
    float* partial;       // [unit][cr][StateLayout<64>::SIZE]
    float* state;         // [unit][StateLayout<64>::SIZE]
    bf16_t* sfrag;        // [unit][kSfragPerUnit]
    uint32_t* kpair;      // [unit][32]
    float* vhalf;         // [unit][64]
    bf16_t* wfrag;        // [head][4][ks][3][64] x 4
    const uint32_t* tasks;       // the queues one after the other
    const uint32_t* queue_off;   // [kStreamQueues + 1]
    uint32_t* counters;
    int units, heads, N, H, W;
    int strips, spc;      // 16-column strips per row, 4-row steps per strip column
    int cr, r_chunk;      // reduce chunks per unit, tokens per chunk
    int ca;               // apply chunks per unit
    int ncs;              // combine slices per unit (0 with cr == 1: the reduce task's result is final)
    int nw;               // weight tasks whose completion pass 2 waits for (0: the table is ready)
    int nw_tasks;         // weight tasks in the lists
    int norm_none, write_state;
    float eps, lin_scale, tscale, unscale;
    TensorStrides in, out_st;
    int spin_limit;
};

__device__ __forceinline__ uint32_t ctr_add(uint32_t* p)
{
    return __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// records the first problem of a launch: code, then two words of detail
__device__ __forceinline__ void stream_error(uint32_t* ctr, uint32_t code, uint32_t d0, uint32_t d1)
{
    if (__hip_atomic_exchange(&ctr[kCtrError], code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        st_agent(&ctr[kCtrError + 1], d0);
        st_agent(&ctr[kCtrError + 2], d1);
    }
}

// thread 0 of a workgroup: poll until *p >= target; false if the wait was given up
__device__ __forceinline__ bool wait_count(uint32_t* ctr, int word, uint32_t target, int limit)
{
    int spins = 0;
    while (ld_agent(&ctr[word]) < target) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > limit || ((spins & 255) == 0 && ld_agent(&ctr[kCtrError]) != 0u)) {
            stream_error(ctr, kStreamErrWait, static_cast<uint32_t>(word), target);
            return false;
        }
    }
    return true;
}

// every store of this wave has been performed before the barrier lets anyone bump a counter
__device__ __forceinline__ void publish_barrier()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// ---------------------------------------------------------------- combine slices
// Sum of `n` partials `stride` floats apart for two entries at once, index order, all loads of
// up to 16 partials of both in flight together.
__device__ __forceinline__ void sum_partials2(const float* p0, const float* p1, int n, size_t stride,
                                              float& s0, float& s1)
{
    s0 = s1 = 0.f;
    for (int sp = 0; sp < n; sp += 16) {
        float t0[16], t1[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const bool in = sp + u < n;
            t0[u] = in ? ld_agent(p0 + (sp + u) * stride) : 0.f;
            t1[u] = in ? ld_agent(p1 + (sp + u) * stride) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (sp + u < n) {
                s0 += t0[u];
                s1 += t1[u];
            }
    }
}

// entry t of kCombineEntries of one unit: fixed-order sums of the partial states into the fp32
// state and the operand tables of pass 2
template <typename X>
__device__ __forceinline__ void combine_entry(int t, int unit, const StreamArgs& a)
{
    using L = StateLayout<64>;
    const float* p = a.partial + static_cast<size_t>(unit) * a.cr * L::SIZE;
    float* st = a.state + static_cast<size_t>(unit) * L::SIZE;
    float s0, s1;
    if (t < 2048) {
        // S: t = ((nt*2 + ks)*64 + lane)*4 + e2 (the B operand order of the 16x16x32 MFMA)
        const int e2 = t & 3, lane = (t >> 2) & 63, ks = (t >> 8) & 1, nt = t >> 9;
        const int i0 = 32 * ks + 8 * (lane >> 4) + 2 * e2;
        const int j = 16 * nt + (lane & 15);
        sum_partials2(p + i0 * 64 + j, p + (i0 + 1) * 64 + j, a.cr, L::SIZE, s0, s1);
        if (a.write_state) {
            st_agent(&st[i0 * 64 + j], s0);
            st_agent(&st[(i0 + 1) * 64 + j], s1);
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(a.sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
        st_agent(&dst[t], X::pack(s0 * a.tscale, s1 * a.tscale));
    } else if (t < 2048 + 128) {
        // f: 0..63 ksum, 64..127 vsum (they follow each other in the state layout)
        const int f = t - 2048;
        sum_partials2(p + L::KSUM + f, p + L::KSUM + f, a.cr, L::SIZE, s0, s1);
        if (a.write_state) st_agent(&st[L::KSUM + f], s0);
        if (f >= 64) st_agent(&a.vhalf[unit * 64 + (f - 64)], 0.5f * s0);
    } else if (t < kCombineEntries) {
        const int i = t - (2048 + 128);  // pair (ksum[2i], ksum[2i+1]) * table scale
        sum_partials2(p + L::KSUM + 2 * i, p + L::KSUM + 2 * i + 1, a.cr, L::SIZE, s0, s1);
        st_agent(&a.kpair[unit * 32 + i], X::pack(s0 * a.tscale, s1 * a.tscale));
    }
}

// entry t of the filter operand table (see dwconv_weight_frag), with device-scope stores
__device__ __forceinline__ void weight_entry(int t, const StreamArgs& a, int ks)
{
    if (t >= a.heads * 4 * ks * 3 * 64) return;
    const int lane = t & 63;
    const int m = (t >> 6) % 3;
    const int dy = (t / (64 * 3)) % ks;
    const int c = (t / (64 * 3 * ks)) & 3;
    const int head = t / (64 * 3 * ks * 4);
    const int ch = 16 * c + (lane >> 2), i = lane & 3;
    const bf16_t* wr = a.w + ((static_cast<size_t>(head) * 64 + ch) * ks + dy) * ks;
    bf16_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int dx = 4 * m - 4 + k - i + ks / 2;
        const int dxc = min(max(dx, 0), ks - 1);
        const bf16_t val = wr[dxc];
        v[k] = (dx == dxc) ? val : static_cast<bf16_t>(0);
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(a.wfrag) + static_cast<size_t>(t) * 2;
    st_agent(&dst[0], static_cast<uint32_t>(v[0]) | (static_cast<uint32_t>(v[1]) << 16));
    st_agent(&dst[1], static_cast<uint32_t>(v[2]) | (static_cast<uint32_t>(v[3]) << 16));
}

// ---------------------------------------------------------------- pass 2 of one chunk
constexpr int kSfNatPitch = 144;                       // token-major staging: bytes per token row
constexpr int kSfNatBytes = 3 * 8 * kSfNatPitch;       // per wave: 3 loads of 8 tokens
constexpr int kSfVtQuad = 544;                         // operand tile: 64 channels x 8 bytes + spread
constexpr int kSfVtRow = 6 * kSfVtQuad;
constexpr int kSfVtBytes = 4 * kSfVtRow;
constexpr int kSfQPitch = 144;                         // q tile [64 tokens][64 features]
constexpr int kSfQBytes = 64 * kSfQPitch;
constexpr int kSfAbBytes = 64 * 8;                     // per token: the two factors of the linear branch
constexpr int kSfOutTokPitch = 20;                     // output tile [row 4][channel 64][token 16 + pad]
constexpr int kSfOutBytes = 4 * 64 * kSfOutTokPitch * 2;
constexpr int kSfNatOff = 0;
constexpr int kSfVtOff = kSfNatOff + 4 * kSfNatBytes;
constexpr int kSfQOff = kSfVtOff + 2 * kSfVtBytes;
constexpr int kSfAbOff = kSfQOff + 2 * kSfQBytes;
constexpr int kSfOutOff = kSfAbOff + 2 * kSfAbBytes;
constexpr int kStreamLdsBytes = kSfOutOff + 2 * kSfOutBytes;
static_assert(kStreamLdsBytes >= reduce_mfma_lds_bytes<64>(), "pass 1 shares the allocation");
static_assert(2 * (kStreamLdsBytes + 64) <= 160 * 1024, "two workgroups per compute unit");
static_assert(16 * kSfNatPitch <= kSfNatBytes, "the staging tile also holds one output row");

__device__ __forceinline__ void lds_only_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint2 lds_tr8(const unsigned char* addr)
{
    typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(addr));
    return __builtin_bit_cast(uint2, r);
}

__device__ __forceinline__ void store16_nt(void* p, const u32x4_t& val)
{
    __builtin_nontemporal_store(val, reinterpret_cast<u32x4_t*>(p));
}

// Steps [g0, g1) of a unit (step = 4 output rows of one 16-column strip; strip-major, then top
// to bottom).  A maximal run inside one strip column is a segment: NCH - 1 stages that only
// bring in V rows, then one step per stage.
struct SegCursor {
    int g_begin, g_end, t, range_end, strip, y0;
    bool live;
    __device__ __forceinline__ void start(int s0, int s1, int spc)
    {
        range_end = s1;
        g_begin = s0;
        strip = s0 / spc;
        g_end = min(s1, (strip + 1) * spc);
        y0 = 4 * (s0 - strip * spc);
        t = 0;
        live = s0 < s1;
    }
    __device__ __forceinline__ void advance(int spc, int nch)
    {
        if (!live) return;
        if (++t == (g_end - g_begin) + nch - 1) {
            if (g_end >= range_end) {
                live = false;
                return;
            }
            g_begin = g_end;
            g_end = min(range_end, g_begin + spc);
            y0 = 0;
            t = 0;
            ++strip;
        }
    }
};

// quad_perm controls of the data-parallel-primitive moves that build the middle view of a
// window row (see apply_chunk)
constexpr int kDppQuad1233 = 1 | (2 << 2) | (3 << 4) | (3 << 6);
constexpr int kDppQuad2222 = 2 | (2 << 2) | (2 << 4) | (2 << 6);

template <int KS, bool LIN, bool DW, typename X>
__device__ __forceinline__ void apply_chunk(const StreamArgs& a, int unit, int g0, int g1,
                                            unsigned char* lds)
{
    constexpr int RAD = KS / 2;
    constexpr int NCH = (KS + 3 + 3) / 4;   // stages until a segment's first output
    constexpr int WR = 4 * NCH;             // input rows kept in registers
    constexpr int NQ = LIN ? 2 : 0;         // q loads per stage and wave (V: 3)
    static_assert(KS - 1 + 3 < WR, "window rows");

    // (opaque to the optimiser: nothing derived from the lane index is kept alive across tasks)
    const int tid = static_cast<int>(opaque_u32(threadIdx.x));
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = a.W, H = a.H, spc = a.spc;
    const uint32_t in_tok = static_cast<uint32_t>(a.in.n) * 2;
    const uint32_t out_tok = static_cast<uint32_t>(a.out_st.n) * 2;
    const int head = unit % a.heads;
    const bf16_t* qb = wave_uniform(a.q + unit_offset(unit, a.heads, a.in));
    const bf16_t* vb = wave_uniform(a.v + unit_offset(unit, a.heads, a.in));
    unsigned char* ob = reinterpret_cast<unsigned char*>(a.out + unit_offset(unit, a.heads, a.out_st));

    unsigned char* const nat = lds + kSfNatOff + w * kSfNatBytes;

    int n_stages = 0;
    for (int gb = g0; gb < g1;) {
        const int ge = min(g1, (gb / spc + 1) * spc);
        n_stages += (ge - gb) + NCH - 1;
        gb = ge;
    }
    if (n_stages == 0) return;

    // ---- lane roles
    const int tok8 = lane >> 3, oct = lane & 7;        // loads: token of the 8, 16-byte piece of its row
    const int blk = lane >> 2, j = lane & 3;           // convolution: channel 16 w + blk, quad j
    const int ch_dw = 16 * w + blk;
    // staging of V: token-major write, transposing read (token 4 qd + (lane/4)%4, channels
    // 16 (lane/16) + 4 (lane%4)..+3); afterwards lane l holds channel l, the 4 tokens of quad qd
    unsigned char* const nat_wr = nat + tok8 * kSfNatPitch + oct * 16;
    const unsigned char* const nat_rd =
        nat + ((lane >> 2) & 3) * kSfNatPitch + (16 * (lane >> 4) + 4 * (lane & 3)) * 2;
    const int vt_rd = j * kSfVtQuad + ch_dw * 8;
    // stores: see store_row
    const int fl_off = (((lane >> 2) & 3) * kSfOutTokPitch + 4 * (lane & 3)) * 2;
    unsigned char* const orow_wr = nat + (lane & 15) * kSfNatPitch + (lane >> 4) * 16;
    const unsigned char* const orow_rd = nat + (lane >> 3) * kSfNatPitch + (lane & 7) * 16;
    // this wave's V items of a stage (of 4 rows x 3 groups of 8 columns) and q items (4 rows x 2)
    int v_r[3], v_c[3], q_r[2], q_h[2];
#pragma unroll
    for (int it = 0; it < 3; ++it) {
        v_r[it] = (w + 4 * it) / 3;
        v_c[it] = (w + 4 * it) % 3;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        q_r[it] = (w + 4 * it) >> 1;
        q_h[it] = (w + 4 * it) & 1;
    }

    // ---- operands of the unit
    s16x4_t tw[KS][3];
    float bias_dw = 0.f;
    if constexpr (DW) {
        const uint32_t* wf = reinterpret_cast<const uint32_t*>(a.wfrag) +
                             ((static_cast<size_t>(head) * 4 + w) * KS * 3 * 64 + lane) * 2;
#pragma unroll
        for (int dy = 0; dy < KS; ++dy)
#pragma unroll
            for (int m = 0; m < 3; ++m) {
                uint2 e;
                e.x = ld_agent(wf + (dy * 3 + m) * 128);
                e.y = ld_agent(wf + (dy * 3 + m) * 128 + 1);
                tw[dy][m] = __builtin_bit_cast(s16x4_t, e);
            }
        bias_dw = a.bias ? X::one(a.bias[head * 64 + ch_dw]) : 0.f;
    }
    u32x4_t sf[2];
    uint32_t ksw[4];
    float vh = 0.f;
    if constexpr (LIN) {
        const uint32_t* s4 = reinterpret_cast<const uint32_t*>(a.sfrag + static_cast<size_t>(unit) * kSfragPerUnit);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e) sf[ks][e] = ld_agent(s4 + ((w * 2 + ks) * 64 + lane) * 4 + e);
#pragma unroll
        for (int e = 0; e < 4; ++e) ksw[e] = ld_agent(a.kpair + unit * 32 + oct * 4 + e);
        vh = ld_agent(a.vhalf + unit * 64 + 16 * w + (lane & 15));
    }
    const float inv_eps = 1.0f / a.eps, half_n = 0.5f * static_cast<float>(a.N);
    // last 16-byte piece of the unit in q / v and in out: every offset is held below these, so
    // that a mistake in the index arithmetic shows as an error code, not as a memory fault
    const uint32_t in_last = static_cast<uint32_t>(a.N - 1) * in_tok + 112u;
    const uint32_t out_last = static_cast<uint32_t>(a.N - 1) * out_tok + 112u;
    auto checked = [&](uint32_t off) {
        if (off > in_last) {
            stream_error(a.counters, kStreamErrLoad, static_cast<uint32_t>(unit), off);
            off = static_cast<uint32_t>(oct) * 16u;
        }
        return off;
    };

    // Window of the last WR input rows.  Per row a lane keeps quad j (view 0) and quad j + 2
    // (view 2) of the 6 quads of the 24 columns; quad j + 1 (view 1) is put together when it is
    // used: lanes j < 3 take view 0 of lane j + 1, lane 3 takes view 2 of lane 2.
    uint2 win0[WR], win2[WR];
#pragma unroll
    for (int i = 0; i < WR; ++i) win0[i] = win2[i] = make_uint2(0u, 0u);
    auto mid_word = [&](uint32_t v0, uint32_t v2) {
        const uint32_t x = __builtin_amdgcn_update_dpp(0u, v0, kDppQuad1233, 0xf, 0xf, false);
        const uint32_t y = __builtin_amdgcn_update_dpp(0u, v2, kDppQuad2222, 0xf, 0xf, false);
        return j == 3 ? y : x;
    };

    u32x4_t vreg[3], qreg[2];
    uint32_t lmask = 0u;   // bits 0..2: V item inside the grid, bits 4..5: q item valid
    // first column, first output row and 'has output rows' of the stage loaded / staged / in the
    // LDS buffers / in the output tile
    int ld_xs0 = 0, ld_yo = 0, next_xs0 = 0, next_yo = 0, cur_xs0 = 0, cur_yo = 0, prev_xs0 = 0, prev_yo = 0;
    bool ld_comp = false, next_comp = false, cur_comp = false, prev_comp = false;
    SegCursor ld;

    // loads of the cursor's stage; past the end, and for q in the priming stages, every lane
    // reads the unit's first row (one line, never used): every stage issues the same number of
    // loads
    auto issue = [&]() {
        const int xs0 = ld.strip * 16;
        const int rowbase = ld.y0 - RAD + 4 * ld.t;
        const int yo = ld.y0 + 4 * (ld.t - (NCH - 1));
        const bool comp = ld.live && ld.t >= NCH - 1;
        uint32_t mask = 0;
        if constexpr (DW) {
#pragma unroll
            for (int it = 0; it < 3; ++it) {
                const int gy = rowbase + v_r[it], gx = xs0 - 4 + 8 * v_c[it] + tok8;
                const bool ok = ld.live && gy >= 0 && gy < H && gx >= 0 && gx < W;
                if (ok) mask |= 1u << it;
                const uint32_t off = ok ? static_cast<uint32_t>(gy * W + gx) * in_tok + oct * 16 : oct * 16;
                async_load16(vreg[it], vb, checked(off));
            }
        }
        if constexpr (LIN) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int y = yo + q_r[it], x = xs0 + 8 * q_h[it] + tok8;
                const bool ok = comp && y < H && x < W;
                if (ok) mask |= 16u << it;
                const uint32_t off = ok ? static_cast<uint32_t>(y * W + x) * in_tok + oct * 16 : oct * 16;
                async_load16_stream(qreg[it], qb, checked(off));
            }
        }
        lmask = mask;
        ld_xs0 = xs0;
        ld_yo = yo;
        ld_comp = comp;
        ld.advance(spc, NCH);
    };

    // the loaded stage to the LDS buffers of parity `par`
    auto fill = [&](int par) {
        const uint32_t mask = lmask;
        const u32x4_t zero = {0u, 0u, 0u, 0u};
        if constexpr (DW) {
            wait_async_loads<NQ>(vreg[0], vreg[1], vreg[2]);
#pragma unroll
            for (int it = 0; it < 3; ++it)
                *reinterpret_cast<u32x4_t*>(nat_wr + it * 8 * kSfNatPitch) =
                    ((mask >> it) & 1u) ? vreg[it] : zero;
        }
        if constexpr (LIN) {
            wait_async_loads<0>(qreg[0], qreg[1]);
            unsigned char* qt = lds + kSfQOff + par * kSfQBytes;
            float* ab = reinterpret_cast<float*>(lds + kSfAbOff + par * kSfAbBytes);
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const u32x4_t raw = ((mask >> (4 + it)) & 1u) ? qreg[it] : zero;
                float ss = 0.f, dk = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ss = X::dot2(raw[e], raw[e], ss);
                    dk = X::dot2(raw[e], ksw[e], dk);
                }
                ss = row_group_sum<8>(ss);
                dk = row_group_sum<8>(dk);
                // 1 / max(|q|, eps) with the hardware reciprocal square root (1 ulp)
                float inv = fminf(__builtin_amdgcn_rsqf(ss), inv_eps);
                if constexpr (X::kHalf) inv *= a.unscale;  // the tables are scaled down
                float alpha, beta;
                if (a.norm_none) {
                    alpha = inv * a.lin_scale;
                    beta = a.lin_scale;
                } else {
                    beta = __builtin_amdgcn_rcpf(half_n + inv * dk);
                    alpha = inv * beta;
                }
                const int tok = q_r[it] * 16 + q_h[it] * 8 + tok8;
                *reinterpret_cast<u32x4_t*>(qt + tok * kSfQPitch + oct * 16) = raw;
                if (oct == 0) *reinterpret_cast<float2*>(ab + 2 * tok) = make_float2(alpha, beta);
            }
        }
        if constexpr (DW) {
            // the staging tile is private to this wave and LDS operations of one wave complete in
            // issue order: no barrier between its writes and the reads
            __builtin_amdgcn_wave_barrier();
            unsigned char* vt = lds + kSfVtOff + par * kSfVtBytes;
            uint2 u[3][2];
#pragma unroll
            for (int it = 0; it < 3; ++it)
#pragma unroll
                for (int qd = 0; qd < 2; ++qd)
                    u[it][qd] = lds_tr8(nat_rd + (it * 8 + qd * 4) * kSfNatPitch);
#pragma unroll
            for (int it = 0; it < 3; ++it)
#pragma unroll
                for (int qd = 0; qd < 2; ++qd)
                    *reinterpret_cast<uint2*>(vt + v_r[it] * kSfVtRow + (2 * v_c[it] + qd) * kSfVtQuad +
                                              lane * 8) = u[it][qd];
            __builtin_amdgcn_wave_barrier();
        }
        next_xs0 = ld_xs0;
        next_yo = ld_yo;
        next_comp = ld_comp;
    };

    // output row w of the tile of parity `par` (the stage before the current one): transposing read
    // ([channel][token] -> lane = token lane % 16, 8 channels), a wave-private token-major copy,
    // then stores in which every instruction writes 8 whole 128-byte lines
    auto store_row = [&](int par) {
        if (!prev_comp) return;
        const unsigned char* ot = lds + kSfOutOff + par * kSfOutBytes;
        uint2 f_lo[2], f_hi[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int o8 = (lane >> 4) + 4 * it;
            const unsigned char* src = ot + (w * 64 + 8 * o8) * (kSfOutTokPitch * 2) + fl_off;
            f_lo[it] = lds_tr8(src);
            f_hi[it] = lds_tr8(src + 4 * kSfOutTokPitch * 2);
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const u32x4_t val = {f_lo[it].x, f_lo[it].y, f_hi[it].x, f_hi[it].y};
            *reinterpret_cast<u32x4_t*>(orow_wr + it * 64) = val;
        }
        __builtin_amdgcn_wave_barrier();
        u32x4_t line[2];
#pragma unroll
        for (int it = 0; it < 2; ++it)
            line[it] = *reinterpret_cast<const u32x4_t*>(orow_rd + it * 8 * kSfNatPitch);
        __builtin_amdgcn_wave_barrier();
        const int y = prev_yo + w;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int x = prev_xs0 + tok8 + 8 * it;
            if (y >= 0 && y < H && x >= 0 && x < W) {
                const uint32_t off = static_cast<uint32_t>(y * W + x) * out_tok + oct * 16;
                if (off <= out_last) store16_nt(ob + off, line[it]);
                else stream_error(a.counters, kStreamErrStore, static_cast<uint32_t>(unit), off);
            }
        }
    };

    // the current stage, whose data sits in the LDS buffers of parity `par`
    auto consume = [&](int par) {
        if constexpr (DW) {
            const unsigned char* vt = lds + kSfVtOff + par * kSfVtBytes + vt_rd;
#pragma unroll
            for (int i = 0; i + 4 < WR; ++i) {
                win0[i] = win0[i + 4];
                win2[i] = win2[i + 4];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                win0[WR - 4 + r] = *reinterpret_cast<const uint2*>(vt + r * kSfVtRow);
                win2[WR - 4 + r] = *reinterpret_cast<const uint2*>(vt + r * kSfVtRow + 2 * kSfVtQuad);
            }
        }
        if (!cur_comp) return;

        f32x4_t acc[4];
        if constexpr (LIN) {
            const unsigned char* qt = lds + kSfQOff + par * kSfQBytes;
            const float* ab = reinterpret_cast<const float*>(lds + kSfAbOff + par * kSfAbBytes);
            const int g = lane >> 4;
            const int src_lane4 = (16 * j + blk) * 4;  // where the convolution's lane finds its value
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const unsigned char* qrow = qt + (rr * 16 + (lane & 15)) * kSfQPitch + g * 16;
                const u32x4_t a0 = *reinterpret_cast<const u32x4_t*>(qrow);
                const u32x4_t a1 = *reinterpret_cast<const u32x4_t*>(qrow + 64);
                const float4 f0 = *reinterpret_cast<const float4*>(ab + 2 * (rr * 16 + 4 * g));
                const float4 f1 = *reinterpret_cast<const float4*>(ab + 2 * (rr * 16 + 4 * g) + 4);
                const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
                f32x4_t p = X::mfma16(a0, sf[0], z);
                p = X::mfma16(a1, sf[1], p);
                // rows 4 g + r of the product: tokens 4 g + r of the row, channel 16 w + lane % 16
                float o[4];
                o[0] = fmaf(f0.x, p[0], f0.y * vh);
                o[1] = fmaf(f0.z, p[1], f0.w * vh);
                o[2] = fmaf(f1.x, p[2], f1.y * vh);
                o[3] = fmaf(f1.z, p[3], f1.w * vh);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[rr][r] = __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane4, __float_as_int(o[r]))) +
                                 bias_dw;
            }
        } else {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[rr][0] = acc[rr][1] = acc[rr][2] = acc[rr][3] = bias_dw;
        }
        if constexpr (DW) {
            // window row i holds input row (first output row - RAD + i); it meets output row rr
            // with filter row dy = i - rr
#pragma unroll
            for (int i = 0; i < KS + 3; ++i) {
                const uint2 mid = make_uint2(mid_word(win0[i].x, win2[i].x), mid_word(win0[i].y, win2[i].y));
                const s16x4_t b0 = __builtin_bit_cast(s16x4_t, win0[i]);
                const s16x4_t b1 = __builtin_bit_cast(s16x4_t, mid);
                const s16x4_t b2 = __builtin_bit_cast(s16x4_t, win2[i]);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int dy = i - rr;
                    if (dy >= 0 && dy < KS) {
                        acc[rr] = X::mfma4(tw[dy][0], b0, acc[rr]);
                        acc[rr] = X::mfma4(tw[dy][1], b1, acc[rr]);
                        acc[rr] = X::mfma4(tw[dy][2], b2, acc[rr]);
                    }
                }
            }
        }
        unsigned char* ot = lds + kSfOutOff + par * kSfOutBytes;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            uint2 o;
            o.x = X::pack(acc[rr][0], acc[rr][1]);
            o.y = X::pack(acc[rr][2], acc[rr][3]);
            *reinterpret_cast<uint2*>(ot + ((rr * 64 + ch_dw) * kSfOutTokPitch + 4 * j) * 2) = o;
        }
    };

    ld.start(g0, g1, spc);
    issue();   // stage 0
    fill(0);
    cur_xs0 = next_xs0;
    cur_yo = next_yo;
    cur_comp = next_comp;
    issue();   // stage 1
    lds_only_barrier();
    for (int s = 0; s < n_stages; ++s) {
        const int par = s & 1;
        if (s + 1 < n_stages) fill(par ^ 1);   // stage s + 1
        issue();                               // stage s + 2
        store_row(par ^ 1);                    // stage s - 1
        consume(par);                          // stage s
        prev_xs0 = cur_xs0;
        prev_yo = cur_yo;
        prev_comp = cur_comp;
        cur_xs0 = next_xs0;
        cur_yo = next_yo;
        cur_comp = next_comp;
        lds_only_barrier();
    }
    store_row((n_stages - 1) & 1);
    // drain the loads issued past the end before the registers die
    if constexpr (DW) wait_async_loads<0>(vreg[0], vreg[1], vreg[2]);
    if constexpr (LIN) wait_async_loads<0>(qreg[0], qreg[1]);
}

// ---------------------------------------------------------------- the kernel
// grid = a multiple of kStreamQueues (two workgroups per compute unit), block = 256,
// dynamic LDS = kStreamLdsBytes.
template <int KS, bool LIN, bool DW, typename X>
__global__ __launch_bounds__(256, 2) void stream_forward_kernel(StreamArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ uint32_t s_word[2];
    using L = StateLayout<64>;
    const int qx = blockIdx.x % kStreamQueues;
    uint32_t* ctr = a.counters;
    const uint32_t q_begin = a.queue_off[qx], q_len = a.queue_off[qx + 1] - q_begin;

    for (;;) {
        // (opaque to the optimiser: nothing derived from the thread index stays alive across tasks)
        const int tid = static_cast<int>(opaque_u32(threadIdx.x));
        if (tid == 0) {
            const uint32_t t = ctr_add(&ctr[kCtrHead + 32 * qx]);
            s_word[0] = t < q_len ? a.tasks[q_begin + t] : kTaskNone;
        }
        __syncthreads();
        const uint32_t task = __builtin_amdgcn_readfirstlane(s_word[0]);
        __syncthreads();
        if (task == kTaskNone) break;
        const uint32_t kind = task >> 28;
        const int unit = (task >> 12) & 0xffff, chunk = task & 0xfff;
        {
            const int chunks = kind == kTaskWeights ? a.nw_tasks : kind == kTaskReduce ? a.cr
                               : kind == kTaskCombine ? a.ncs : a.ca;
            if (kind > kTaskApply || unit >= a.units || chunk >= chunks) {  // uniform per workgroup
                if (tid == 0) stream_error(ctr, kStreamErrTask, task, static_cast<uint32_t>(qx));
                continue;
            }
        }

        if (kind == kTaskWeights) {
            if constexpr (DW) {
                if (a.nw > 0) {  // (else the registered table is used as it is)
                    for (int e = tid; e < kWeightEntriesPerTask; e += 256)
                        weight_entry(chunk * kWeightEntriesPerTask + e, a, KS);
                    publish_barrier();
                    if (tid == 0) ctr_add(&ctr[kCtrWeights]);
                }
            }
        } else if (kind == kTaskReduce) {
            if constexpr (LIN) {
                ReduceExtras ex = {};
                float* part = a.partial + (static_cast<size_t>(unit) * a.cr + chunk) * L::SIZE;
                if (a.cr == 1) {  // the chunk is the unit: its result is final
                    ex.state = a.state;
                    ex.sfrag = a.sfrag;
                    ex.vhalf = a.vhalf;
                    ex.kpair = a.kpair;
                    ex.tscale = a.tscale;
                    ex.write_state = a.write_state;
                    part = nullptr;
                }
                const int n0 = chunk * a.r_chunk;
#ifndef STREAM_NO_REDUCE
                reduce_mfma_block<64, X, false>(a.k, a.v, part, a.N, n0, min(a.N, n0 + a.r_chunk), a.eps,
                                                a.heads, a.in, ex, unit, lds);
#endif
                publish_barrier();
                if (tid == 0) ctr_add(&ctr[kCtrUnit + 2 * unit + (a.cr == 1 ? 1 : 0)]);
            }
        } else if (kind == kTaskCombine) {
            if constexpr (LIN) {
                if (tid == 0) s_word[1] = wait_count(ctr, kCtrUnit + 2 * unit, a.cr, a.spin_limit) ? 1u : 0u;
                __syncthreads();
                const bool ok = __builtin_amdgcn_readfirstlane(s_word[1]) != 0u;
                if (ok)
                    for (int t = chunk * 256 + tid; t < kCombineEntries; t += a.ncs * 256)
                        combine_entry<X>(t, unit, a);
                publish_barrier();
                if (tid == 0) ctr_add(&ctr[kCtrUnit + 2 * unit + 1]);
            }
        } else {
            if (tid == 0) {
                bool ok = true;
                if (LIN) ok = wait_count(ctr, kCtrUnit + 2 * unit + 1, a.ncs > 0 ? a.ncs : 1, a.spin_limit);
                if (DW && ok && a.nw > 0) ok = wait_count(ctr, kCtrWeights, a.nw, a.spin_limit);
                s_word[1] = ok ? 1u : 0u;
            }
            __syncthreads();
            if (__builtin_amdgcn_readfirstlane(s_word[1]) != 0u) {
                const int steps = a.strips * a.spc;
                const int g0 = static_cast<int>(static_cast<long long>(chunk) * steps / a.ca);
                const int g1 = static_cast<int>(static_cast<long long>(chunk + 1) * steps / a.ca);
                apply_chunk<KS, LIN, DW, X>(a, unit, g0, g1, lds);
            }
            __syncthreads();
        }
    }

    // the last workgroup to leave clears the counters for the next launch (the error word stays)
    const int tid = threadIdx.x;
    if (tid == 0) s_word[1] = ctr_add(&ctr[kCtrDone]) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (__builtin_amdgcn_readfirstlane(s_word[1]) != 0u) {
        const int n = static_cast<int>(stream_counter_words(a.units));
        for (int i = tid; i < n; i += 256)
            if (i != kCtrError) st_agent(&ctr[i], 0u);
    }
}

}  // namespace castling
