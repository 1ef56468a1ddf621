// C ABI of the linear-angular attention layer: argument checks, workspace,
// kernel dispatch.  See include/castling_attn.h for the contract.
#include "../../include/castling_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cfloat>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>

#include "apply_generic.hpp"
#include "apply_mfma.hpp"
#include "backward.hpp"
#include "common.hpp"
#include "fused_small.hpp"
#include "pairwise.hpp"
#include "reduce_generic.hpp"
#include "reduce_mfma.hpp"

using namespace castling;

// Scratch memory of castling_attn_forward_static: one copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[CASTLING_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kTargetReduceBlocks = 256;  // one block per compute unit
constexpr int kMinChunkTokens = 128;

thread_local char g_hip_error[256] = "HIP runtime error";

int hip_fail(hipError_t e)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "HIP runtime error: %s", hipGetErrorString(e));
    return CASTLING_ERR_HIP;
}

#define HIP_TRY(expr)                              \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return hip_fail(e_); \
    } while (0)

constexpr size_t kMaxLdsBytes = 160 * 1024;  // LDS of one compute unit

size_t dtype_size(int dt) { return dt == CASTLING_F32 ? 4 : 2; }

// f(T{}, integral_constant<int, D>{}) for the handle's I/O type and head width
template <typename F>
auto dispatch_type_width(int dtype, int d, F&& f)
{
    auto with_t = [&](auto t) {
        switch (d) {
            case 16: return f(t, std::integral_constant<int, 16>{});
            case 32: return f(t, std::integral_constant<int, 32>{});
            case 64: return f(t, std::integral_constant<int, 64>{});
            default: return f(t, std::integral_constant<int, 128>{});
        }
    };
    if (dtype == CASTLING_F32) return with_t(float{});
    if (dtype == CASTLING_F16) return with_t(f16_t{});
    return with_t(bf16_t{});
}
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// What one apply launch covers: the grid with the handle's branches and filter size, or the
// tokens in front of the grid as a 1 x extra "grid" with the linear branch only.
struct ApplyView {
    int grid_h, grid_w, ks;
    uint32_t branches;
};

// Bytes of the parts of a handle's workspace, in the order they lie in it (wfrag twice).
struct WorkspaceParts {
    size_t partial, state, sfrag, kfrag, vhalf, wfrag, a, kbp, kb, wflip, fpart;
};

struct castling_attn {
    castling_attn_desc_t desc;
    WorkspaceParts parts;
    ApplyView view;     // read by the apply launchers
    int device;
    int units;
    int n_split;
    int chunk;
    TensorStrides in_st, out_st;  // element strides of q/k/v and of out (defaults resolved)
    TensorStrides q_st;           // of q: in_st, or its own where the queries are pooled
    size_t in_span, out_span;     // bytes from the first to one past the last element addressed
    size_t q_span;
    int pool;                     // stride of the queries on the token grid (1 or 2)
    int qgrid_h, qgrid_w, nq;     // grid and count of the queries (= of the rows of out)
    bool residual_q;
    int dpad;           // width the kernels run at: 16 / 32 / 64 / 128, narrower heads zero-padded
    int state_size;     // floats per unit (of width dpad)
    bool mfma_reduce;   // bf16 / fp16, d = 32 or 64: K_hat^T V on the matrix cores
    bool mfma_apply;    // bf16 / fp16, d = 64: q.S and the DWConv on the matrix cores
    bool half16;        // the 16-bit format is fp16 (else bf16)
    bool pair;          // d = 32: pass 2 runs two heads as one 64-channel unit (mfma_apply is set)
    bool pair_reduce;   // ... and so does pass 1: the heads are neighbours in memory (whole rows)
    int apply_units, apply_heads;         // units and heads as pass 2 counts them
    TensorStrides apply_in, apply_out;    // strides of those units
    uint32_t in_skew, out_skew;           // pair: see ApplyMfmaParams
    bool fused;         // forward() runs the one-kernel path (small N)
    bool state_valid;   // the workspace holds the state of the last reduce
    bool apply_ready;   // the workspace holds what apply() needs (state / tables / partials)
    bool sum_in_apply;  // forward(): the vector-ALU apply sums the partial states itself (no combine)
    bool partials_pending;  // set by a reduce that left the combine to the apply launch
    int num_cus;        // compute units of the device
    size_t apply_lds;   // dynamic LDS of the apply kernel
    // workspace (one allocation)
    unsigned char* workspace;
    size_t workspace_bytes;
    float* partial;     // [units][n_split][state_size]
    float* state;       // [units][state_size]
    bf16_t* sfrag;      // MFMA path: operand tables, see apply_mfma.hpp
    bf16_t* kfrag;
    float* vhalf;
    bf16_t* wfrag;      // filter operand table of the call in progress (rebuilt by every call that passes filters)
    bf16_t* wfrag_reg;  // filter operand table of castling_attn_prepare_weights; nothing else writes it
    const void* prepared_w;  // filters registered by castling_attn_prepare_weights
    bool use_registered;     // the apply launch in progress reads wfrag_reg
    // The backward pass runs pass 2 on other tensors: q := k, v := g (layout of out), out := dv
    // (layout of v), without the normaliser.  generic: on the vector-ALU kernel even where the
    // handle's pass 2 is on the matrix cores (the layouts of v and out differ).
    struct {
        bool on, generic;
        TensorStrides q, v, out;
        float lin_scale;  // factor on the linear branch (the state of (q, a) is scaled, see backward.hpp)
    } ov;
    // backward workspace (CASTLING_FLAG_TRAINING; part of the one allocation)
    bool training;
    void* a_buf;        // a_t = dLoss/dnum_t, I/O type, layout and span of q
    float* kb_part;     // [units][row tiles][dpad]
    float* kb;          // [units][dpad]
    void* wflip;        // filters turned by 180 degrees
    float* fpart;       // [units][filter chunks][ks*ks + 1][dpad]
    int row_tiles, qrow_tiles, filter_chunks;  // 64-row tiles of the tokens / of the queries
    void* q_up;         // q_pool = 2: q and g on their places in the fine grid (layout of k, v;
    void* g_up;         //   zero elsewhere, like a_buf), see BwdRowsParams
    bool mfma_rows;     // dq / dk on the matrix cores (16-bit, d = 32 or 64)
    int kb_parts;       // shares of kb' per unit
};

namespace {

// ------------------------------------------------------------------ reduce
template <typename T, int D>
void launch_reduce_generic(castling_attn* h, const void* k, const void* v, hipStream_t s)
{
    hipLaunchKernelGGL((reduce_generic_kernel<T, D>), dim3(h->n_split, h->units), dim3(256), 0, s,
                       static_cast<const T*>(k), static_cast<const T*>(v), h->partial, h->desc.N,
                       h->n_split, h->chunk, h->desc.eps, h->desc.heads, h->in_st, h->desc.d);
}

// w != nullptr: extra grid rows build the DWConv weight operand table.
// direct: the blocks' results are final (n_split == 1); they write state and tables themselves.
// PAIR: the units are the pairs of 32-wide heads pass 2 works on.
template <int D, typename X, bool PAIR = false>
void launch_reduce_mfma(castling_attn* h, const void* k, const void* v, const void* w, bool direct,
                        hipStream_t s)
{
    const int units = PAIR ? h->apply_units : h->units;
    const int heads = PAIR ? h->apply_heads : h->desc.heads;
    ReduceExtras ex = {};
    ex.state = direct ? h->state : nullptr;
    ex.sfrag = h->sfrag;
    ex.kfrag = h->kfrag;
    ex.vhalf = h->vhalf;
    ex.w = static_cast<const bf16_t*>(w);
    ex.wfrag = h->wfrag;
    ex.units = units;
    ex.heads = heads;
    ex.ks = h->desc.dw_kernel;
    ex.tscale = X::table_scale(h->desc.N);
    ex.pair_skew = h->in_skew;
    const int per_row = h->n_split * 64 * kReduceWaves;
    const int wthreads = heads * 4 * ex.ks * 3 * 64;
    const int wrows = w ? (wthreads + per_row - 1) / per_row : 0;
    hipLaunchKernelGGL((reduce_mfma_kernel<D, X, PAIR>), dim3(h->n_split, units + wrows),
                       dim3(64 * kReduceWaves), 0, s, static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), h->partial, h->desc.N, h->n_split, h->chunk,
                       h->desc.eps, heads, PAIR ? h->apply_in : h->in_st, ex);
}

template <int D>
void launch_combine(castling_attn* h, hipStream_t s)
{
    using L = StateLayout<D>;
    hipLaunchKernelGGL((combine_kernel<D>), dim3((L::SIZE + 255) / 256, h->units), dim3(256), 0, s,
                       h->partial, h->state, h->n_split);
}

// w != nullptr: also prepare the DWConv weight operands of the MFMA apply kernel
// defer_combine: leave the partial states as they are for an apply launch that sums them
int do_reduce(castling_attn* h, const void* k, const void* v, const void* w, hipStream_t s,
              bool defer_combine = false)
{
    const int d = h->dpad;
    h->state_valid = true;
    h->apply_ready = true;
    h->partials_pending = false;
    // with one split per unit the reduce kernel's result is final: it writes the state and
    // the apply kernel's operand tables itself, and no combine is launched
    const bool direct = h->mfma_apply && !h->pair && h->n_split == 1;
    if (h->mfma_reduce) {
        if (h->half16) {
            if (h->pair_reduce) launch_reduce_mfma<64, F16Fmt, true>(h, k, v, nullptr, false, s);
            else if (d == 32) launch_reduce_mfma<32, F16Fmt>(h, k, v, nullptr, false, s);
            else launch_reduce_mfma<64, F16Fmt>(h, k, v, direct ? w : nullptr, direct, s);
        } else {
            if (h->pair_reduce) launch_reduce_mfma<64, Bf16Fmt, true>(h, k, v, nullptr, false, s);
            else if (d == 32) launch_reduce_mfma<32, Bf16Fmt>(h, k, v, nullptr, false, s);
            else launch_reduce_mfma<64, Bf16Fmt>(h, k, v, direct ? w : nullptr, direct, s);
        }
    } else {
        dispatch_type_width(h->desc.io_dtype, d, [&](auto t, auto dc) {
            launch_reduce_generic<decltype(t), decltype(dc)::value>(h, k, v, s);
            return 0;
        });
    }
    HIP_TRY(hipGetLastError());
    if (direct) return CASTLING_OK;
    // vector-ALU apply with one split per unit: the partial layout is the state layout and the
    // handle points `partial` at `state`, so the reduce kernel's result is final as written
    if (!h->mfma_apply && h->n_split == 1) return CASTLING_OK;
    if (defer_combine) {
        h->state_valid = false;
        h->partials_pending = true;
        return CASTLING_OK;
    }
    if (h->pair) {
        const int gx = (kCombineFragThreads + 255) / 256;
        const int ks = h->desc.dw_kernel;
        const int wthreads = h->apply_heads * 4 * ks * 3 * 64;
        const int wrows = w ? (wthreads + gx * 256 - 1) / (gx * 256) : 0;
        if (h->half16)
            hipLaunchKernelGGL(combine_pair_frag_kernel<F16Fmt>, dim3(gx, h->apply_units + wrows),
                               dim3(256), 0, s, h->partial, h->state, h->sfrag, h->kfrag, h->vhalf,
                               h->n_split, h->apply_units, h->pair_reduce ? 1 : 0,
                               static_cast<const bf16_t*>(w), h->wfrag, h->apply_heads, ks,
                               F16Fmt::table_scale(h->desc.N));
        else
            hipLaunchKernelGGL(combine_pair_frag_kernel<Bf16Fmt>, dim3(gx, h->apply_units + wrows),
                               dim3(256), 0, s, h->partial, h->state, h->sfrag, h->kfrag, h->vhalf,
                               h->n_split, h->apply_units, h->pair_reduce ? 1 : 0,
                               static_cast<const bf16_t*>(w), h->wfrag, h->apply_heads, ks,
                               Bf16Fmt::table_scale(h->desc.N));
    } else if (h->mfma_apply) {
        const int gx = (kCombineFragThreads + 255) / 256;
        const int ks = h->desc.dw_kernel;
        const int wthreads = h->desc.heads * 4 * ks * 3 * 64;
        const int wrows = w ? (wthreads + gx * 256 - 1) / (gx * 256) : 0;
        if (h->half16)
            hipLaunchKernelGGL(combine_frag_kernel<F16Fmt>, dim3(gx, h->units + wrows), dim3(256), 0,
                               s, h->partial, h->state, h->sfrag, h->kfrag, h->vhalf, h->n_split,
                               h->units, static_cast<const bf16_t*>(w), h->wfrag, h->desc.heads, ks,
                               F16Fmt::table_scale(h->desc.N));
        else
            hipLaunchKernelGGL(combine_frag_kernel<Bf16Fmt>, dim3(gx, h->units + wrows), dim3(256), 0,
                               s, h->partial, h->state, h->sfrag, h->kfrag, h->vhalf, h->n_split,
                               h->units, static_cast<const bf16_t*>(w), h->wfrag, h->desc.heads, ks,
                               Bf16Fmt::table_scale(h->desc.N));
    } else {
        dispatch_type_width(CASTLING_F32, d, [&](auto, auto dc) {
            launch_combine<decltype(dc)::value>(h, s);
            return 0;
        });
    }
    HIP_TRY(hipGetLastError());
    return CASTLING_OK;
}

// ------------------------------------------------------------------ apply
// launch = false: set the kernel's LDS attribute and record its LDS size (create time)
template <typename T, int D, int KS, int S>
hipError_t apply_generic(castling_attn* h, bool launch, const void* q, const void* v,
                         const void* w, const void* bias, void* out, hipStream_t s)
{
    constexpr size_t lds = apply_generic_lds_bytes<T, D, KS, S>();
    if (!launch) {
        h->apply_lds = lds;
        if (lds > kMaxLdsBytes) return hipSuccess;  // create reports the shape as unsupported
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&apply_generic_kernel<T, D, KS, S>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   static_cast<int>(lds));
    }
    const castling_attn_desc_t& d = h->desc;
    ApplyParams p = {};
    p.N = d.N;
    p.grid_h = h->view.grid_h;
    p.grid_w = h->view.grid_w;
    p.tiles_x = (p.grid_w + kApplyTW - 1) / kApplyTW;
    p.norm_none = h->ov.on || d.norm == CASTLING_NORM_NONE;
    p.do_linear = (h->view.branches & CASTLING_BRANCH_LINEAR) != 0;
    p.do_dwconv = (h->view.branches & CASTLING_BRANCH_DWCONV) != 0;
    p.eps = d.eps;
    p.in = h->ov.on ? h->ov.v : h->in_st;
    p.out = h->ov.on ? h->ov.out : h->out_st;
    p.n_partials = h->partials_pending ? h->n_split : 1;
    p.d_valid = d.d;
    p.qs = h->ov.on ? h->ov.q : h->q_st;
    p.vgrid_h = S == 1 ? p.grid_h : d.grid_h;
    p.vgrid_w = S == 1 ? p.grid_w : d.grid_w;
    p.residual_q = h->residual_q && !h->ov.on;
    p.lin_scale = h->ov.on ? h->ov.lin_scale : 1.0f;
    const int tiles_y = (p.grid_h + kApplyTH - 1) / kApplyTH;
    hipLaunchKernelGGL((apply_generic_kernel<T, D, KS, S>), dim3(p.tiles_x * tiles_y, h->units),
                       dim3(256), lds, s, static_cast<const T*>(q), static_cast<const T*>(v),
                       static_cast<const T*>(w), static_cast<const T*>(bias),
                       h->partials_pending ? h->partial : h->state, static_cast<T*>(out), d.heads, p);
    return hipGetLastError();
}

// w == nullptr: the weight operand table has already been prepared on this stream
template <int KS, bool LIN, bool DW, typename X>
hipError_t apply_mfma_branches(castling_attn* h, bool launch, const void* q, const void* v,
                               const void* w, const void* bias, void* out, hipStream_t s)
{
    // only the linear branch tells a pair of heads from one head
    constexpr bool kPairKernel = LIN;
    const bool pair = kPairKernel && h->pair;
    if (!launch) {
        h->apply_lds = kApplyMfmaLdsBytes;
        const void* fn = reinterpret_cast<const void*>(&apply_mfma_kernel<KS, LIN, DW, X, false>);
        if constexpr (kPairKernel)
            if (pair) fn = reinterpret_cast<const void*>(&apply_mfma_kernel<KS, LIN, DW, X, true>);
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kApplyMfmaLdsBytes);
    }
    const castling_attn_desc_t& d = h->desc;
    ApplyMfmaParams p = {};
    p.N = d.N;
    p.grid_h = h->view.grid_h;
    p.grid_w = h->view.grid_w;
    p.strips = (p.grid_w + kStripW - 1) / kStripW;
    p.norm_none = h->ov.on || d.norm == CASTLING_NORM_NONE;
    p.do_linear = LIN;
    p.do_dwconv = DW;
    p.eps = d.eps;
    p.in = h->apply_in;
    p.out = h->apply_out;
    p.in_skew = h->in_skew;
    p.out_skew = h->out_skew;
    p.lin_scale = h->ov.on ? h->ov.lin_scale : 1.0f;
    if (DW && w) {
        const int threads = h->apply_heads * 4 * KS * 3 * 64;
        hipLaunchKernelGGL(dwconv_weight_frag_kernel, dim3((threads + 255) / 256), dim3(256), 0, s,
                           static_cast<const bf16_t*>(w), h->wfrag, h->apply_heads, KS);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // one persistent block per compute unit; every block takes an equal share of the steps
    const int total_steps = h->apply_units * p.strips * ((p.grid_h + 3) / 4);
    const int blocks = total_steps < h->num_cus ? total_steps : h->num_cus;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(64 * kApplyWaves), kApplyMfmaLdsBytes, s,
                           static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(v),
                           static_cast<const bf16_t*>(bias), h->sfrag, h->kfrag, h->vhalf,
                           h->use_registered ? h->wfrag_reg : h->wfrag,
                           static_cast<bf16_t*>(out), h->apply_heads, total_steps, p);
    };
    if constexpr (kPairKernel) {
        if (pair) go(apply_mfma_kernel<KS, LIN, DW, X, true>);
        else go(apply_mfma_kernel<KS, LIN, DW, X, false>);
    } else {
        go(apply_mfma_kernel<KS, LIN, DW, X, false>);
    }
    return hipGetLastError();
}

template <int KS, typename X>
hipError_t apply_mfma_fmt(castling_attn* h, bool launch, const void* q, const void* v,
                          const void* w, const void* bias, void* out, hipStream_t s)
{
    const bool lin = (h->view.branches & CASTLING_BRANCH_LINEAR) != 0;
    const bool dw = (h->view.branches & CASTLING_BRANCH_DWCONV) != 0;
    if (lin && dw) return apply_mfma_branches<KS, true, true, X>(h, launch, q, v, w, bias, out, s);
    if (lin) return apply_mfma_branches<KS, true, false, X>(h, launch, q, v, w, bias, out, s);
    return apply_mfma_branches<KS, false, true, X>(h, launch, q, v, w, bias, out, s);
}

template <int KS>
hipError_t apply_mfma(castling_attn* h, bool launch, const void* q, const void* v, const void* w,
                      const void* bias, void* out, hipStream_t s)
{
    return h->half16 ? apply_mfma_fmt<KS, F16Fmt>(h, launch, q, v, w, bias, out, s)
                     : apply_mfma_fmt<KS, Bf16Fmt>(h, launch, q, v, w, bias, out, s);
}

template <typename T, int D>
hipError_t apply_generic_ks(castling_attn* h, bool launch, const void* q, const void* v,
                            const void* w, const void* bias, void* out, hipStream_t s)
{
    if (h->pool == 2 && !h->ov.on) {
        switch (h->view.ks) {
            case 1: return apply_generic<T, D, 1, 2>(h, launch, q, v, w, bias, out, s);
            case 3: return apply_generic<T, D, 3, 2>(h, launch, q, v, w, bias, out, s);
            case 5: return apply_generic<T, D, 5, 2>(h, launch, q, v, w, bias, out, s);
            case 7: return apply_generic<T, D, 7, 2>(h, launch, q, v, w, bias, out, s);
            default: return apply_generic<T, D, 9, 2>(h, launch, q, v, w, bias, out, s);
        }
    }
    switch (h->view.ks) {
        case 1: return apply_generic<T, D, 1, 1>(h, launch, q, v, w, bias, out, s);
        case 3: return apply_generic<T, D, 3, 1>(h, launch, q, v, w, bias, out, s);
        case 5: return apply_generic<T, D, 5, 1>(h, launch, q, v, w, bias, out, s);
        case 7: return apply_generic<T, D, 7, 1>(h, launch, q, v, w, bias, out, s);
        default: return apply_generic<T, D, 9, 1>(h, launch, q, v, w, bias, out, s);
    }
}

// one launch for what h->view describes
hipError_t do_apply_view(castling_attn* h, bool launch, const void* q, const void* v, const void* w,
                         const void* bias, void* out, hipStream_t s)
{
    if (h->mfma_apply && !(h->ov.on && h->ov.generic)) {
        switch (h->view.ks) {
            case 1: return apply_mfma<1>(h, launch, q, v, w, bias, out, s);
            case 3: return apply_mfma<3>(h, launch, q, v, w, bias, out, s);
            case 5: return apply_mfma<5>(h, launch, q, v, w, bias, out, s);
            case 7: return apply_mfma<7>(h, launch, q, v, w, bias, out, s);
            default: return apply_mfma<9>(h, launch, q, v, w, bias, out, s);
        }
    }
    return dispatch_type_width(h->desc.io_dtype, h->dpad, [&](auto t, auto dc) {
        return apply_generic_ks<decltype(t), decltype(dc)::value>(h, launch, q, v, w, bias, out, s);
    });
}

// Pass 2 of a unit: the grid tokens with the handle's branches, then the tokens in front of the
// grid (class tokens) with the linear branch alone -- as a 1 x extra grid through the same
// kernels -- or zeros if the linear branch is off.
hipError_t do_apply(castling_attn* h, bool launch, const void* q, const void* v, const void* w,
                    const void* bias, void* out, hipStream_t s)
{
    const castling_attn_desc_t& d = h->desc;
    const int extra = d.extra_tokens;
    const bool lin = (d.branches & CASTLING_BRANCH_LINEAR) != 0;
    // (the backward's pass 2 always runs on the grid of k and v)
    const ApplyView grid_view = {h->ov.on ? d.grid_h : h->qgrid_h, h->ov.on ? d.grid_w : h->qgrid_w,
                                 d.dw_kernel, d.branches};
    const ApplyView extra_view = {1, extra, 1, CASTLING_BRANCH_LINEAR};
    h->view = grid_view;
    if (!launch) {
        hipError_t e = do_apply_view(h, false, q, v, w, bias, out, s);
        if (e == hipSuccess && extra > 0 && lin) {
            const size_t lds = h->apply_lds;
            h->view = extra_view;
            e = do_apply_view(h, false, q, v, w, bias, out, s);
            if (lds > h->apply_lds) h->apply_lds = lds;
            h->view = grid_view;
        }
        return e;
    }
    const size_t es = dtype_size(d.io_dtype);
    auto skip = [&](const void* p, long long tok_stride) -> const void* {
        return p ? static_cast<const unsigned char*>(p) + static_cast<size_t>(extra) * tok_stride * es
                 : nullptr;
    };
    const TensorStrides& out_st = h->ov.on ? h->ov.out : h->out_st;
    hipError_t e = do_apply_view(h, true, skip(q, h->ov.on ? h->ov.q.n : h->q_st.n),
                                 skip(v, h->ov.on ? h->ov.v.n : h->in_st.n), w, bias,
                                 const_cast<void*>(skip(out, out_st.n)), s);
    if (e != hipSuccess || extra == 0) return e;
    if (lin) {
        h->view = extra_view;
        e = do_apply_view(h, true, q, v, nullptr, nullptr, out, s);
        h->view = grid_view;
        return e;
    }
    dispatch_type_width(d.io_dtype, d.d, [&](auto t, auto) {
        using T = decltype(t);
        const int pieces = extra * d.d / IO<T>::VEC;
        hipLaunchKernelGGL(zero_rows_kernel<T>, dim3((pieces + 255) / 256, h->units), dim3(256), 0, s,
                           static_cast<T*>(out), extra, d.d, d.heads, out_st);
        return 0;
    });
    return hipGetLastError();
}

// ------------------------------------------------------------------ backward
// the factor a = dLoss/dnum is stored with (see BwdRowsParams)
float bwd_a_scale(const castling_attn* h)
{
    return h->desc.norm == CASTLING_NORM_NONE ? 1.0f : static_cast<float>(h->desc.N);
}

// launch = false: set the kernels' LDS attributes, record the largest in *lds (create time)
// parameters of a per-row launch: the query side (rows of q, possibly pooled) or the key side
BwdRowsParams bwd_rows_params(const castling_attn* h, bool query)
{
    const castling_attn_desc_t& d = h->desc;
    BwdRowsParams p = {};
    p.N = d.N;
    p.rows = query ? h->nq : d.N;
    p.tiles = query ? h->qrow_tiles : h->row_tiles;
    p.norm_none = d.norm == CASTLING_NORM_NONE;
    p.residual_q = h->residual_q;
    p.d_valid = d.d;
    p.eps = d.eps;
    p.ascale = bwd_a_scale(h);
    p.mscale = query ? kInvPi : kInvPi / p.ascale;
    p.in = h->in_st;
    p.out = h->out_st;
    p.xs = query ? h->q_st : h->in_st;
    if (query && h->pool == 2) {
        p.up_s = 2;
        p.up_wq = h->qgrid_w;
        p.up_w = d.grid_w;
        p.q_up = h->q_up;
        p.g_up = h->g_up;
    }
    return p;
}

template <typename X, int D>
hipError_t bwd_rows_mfma(castling_attn* h, bool launch, bool query, const void* x, const void* y,
                         void* dx, size_t* lds, hipStream_t s, const BwdRowsParams& p)
{
    constexpr size_t bytes = bwd_rows_mfma_lds_bytes<D>();
    if (!launch) {
        if (bytes > *lds) *lds = bytes;
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void*>(&bwd_rows_mfma_kernel<X, D, true>),
            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_rows_mfma_kernel<X, D, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    }
    // the block loads the state once: several tiles per block where there are many
    const long long all = static_cast<long long>(p.tiles) * h->units;
    const int tpb = static_cast<int>(std::max(1ll, std::min(8ll, all / 1024)));
    const dim3 grid((p.tiles + tpb - 1) / tpb, h->units);
    auto u16 = [](const void* ptr) { return static_cast<const uint16_t*>(ptr); };
    if (query)
        hipLaunchKernelGGL((bwd_rows_mfma_kernel<X, D, true>), grid, dim3(256), bytes, s, u16(x), u16(y),
                           h->state, nullptr, static_cast<uint16_t*>(h->a_buf), h->kb_part,
                           static_cast<uint16_t*>(dx), h->desc.heads, p, tpb);
    else
        hipLaunchKernelGGL((bwd_rows_mfma_kernel<X, D, false>), grid, dim3(256), bytes, s, u16(x), u16(y),
                           h->state, h->kb, nullptr, nullptr, static_cast<uint16_t*>(dx),
                           h->desc.heads, p, tpb);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t bwd_rows(castling_attn* h, bool launch, bool query, const void* x, const void* y,
                    void* dx, size_t* lds, hipStream_t s)
{
    if constexpr (sizeof(T) == 2 && (D == 32 || D == 64)) {
        if (h->mfma_rows) {
            const BwdRowsParams p = launch ? bwd_rows_params(h, query) : BwdRowsParams{};
            return h->half16 ? bwd_rows_mfma<F16Fmt, D>(h, launch, query, x, y, dx, lds, s, p)
                             : bwd_rows_mfma<Bf16Fmt, D>(h, launch, query, x, y, dx, lds, s, p);
        }
    }
    constexpr size_t bytes = bwd_rows_lds_bytes<D>();
    if (!launch) {
        if (bytes > *lds) *lds = bytes;
        if (bytes > kMaxLdsBytes) return hipSuccess;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_rows_kernel<T, D, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           static_cast<int>(bytes));
        if (e != hipSuccess) return e;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_rows_kernel<T, D, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    }
    const castling_attn_desc_t& d = h->desc;
    const BwdRowsParams p = bwd_rows_params(h, query);
    const dim3 grid(p.tiles, h->units);
    if (query)
        hipLaunchKernelGGL((bwd_rows_kernel<T, D, true>), grid, dim3(256), bytes, s,
                           static_cast<const T*>(x), static_cast<const T*>(y), h->state, nullptr,
                           static_cast<T*>(h->a_buf), h->kb_part, static_cast<T*>(dx), d.heads, p);
    else
        hipLaunchKernelGGL((bwd_rows_kernel<T, D, false>), grid, dim3(256), bytes, s,
                           static_cast<const T*>(x), static_cast<const T*>(y), h->state, h->kb,
                           nullptr, nullptr, static_cast<T*>(dx), d.heads, p);
    return hipGetLastError();
}

// fills the parameters of a filter-gradient launch; returns the pointers to the first grid token
template <typename T>
BwdFilterParams bwd_filter_params(const castling_attn* h, int tile_rows, const void* v, const void* g,
                                  const T** vg, const T** gg)
{
    const castling_attn_desc_t& d = h->desc;
    BwdFilterParams p = {};
    p.grid_h = d.grid_h;
    p.grid_w = d.grid_w;
    p.tiles_x = (d.grid_w + kApplyTW - 1) / kApplyTW;
    p.n_tiles = p.tiles_x * ((d.grid_h + tile_rows - 1) / tile_rows);
    p.chunks = h->filter_chunks;
    p.d_valid = d.d;
    p.in = h->in_st;
    p.out = h->pool == 2 ? h->in_st : h->out_st;  // (pooled queries: g comes on the fine grid)
    // the class tokens in front of the grid take no part in the convolution
    *vg = static_cast<const T*>(v) + static_cast<long long>(d.extra_tokens) * h->in_st.n;
    *gg = static_cast<const T*>(g) + static_cast<long long>(d.extra_tokens) * p.out.n;
    return p;
}

// 16-bit I/O: the kernel on two-element dot products, where its LDS image fits
template <typename X, int D, int KS>
hipError_t bwd_filter_dot2(castling_attn* h, bool launch, const void* v, const void* g, size_t* lds,
                           hipStream_t s)
{
    constexpr size_t bytes = bwd_filter_dot2_lds_bytes<D, KS>();
    if (!launch) {
        if (bytes > *lds) *lds = bytes;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_filter_dot2_kernel<X, D, KS>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    }
    const uint16_t *vg, *gg;
    const BwdFilterParams p = bwd_filter_params<uint16_t>(h, kApplyTH, v, g, &vg, &gg);
    hipLaunchKernelGGL((bwd_filter_dot2_kernel<X, D, KS>), dim3(h->filter_chunks, h->units),
                       dim3(kBwdFilterThreads), bytes, s, vg, gg, h->fpart, h->desc.heads, p);
    return hipGetLastError();
}

template <typename T, int D, int KS>
hipError_t bwd_filter_ks(castling_attn* h, bool launch, const void* v, const void* g, size_t* lds,
                         hipStream_t s)
{
    constexpr size_t bytes = bwd_filter_lds_bytes<T, D, KS>();
    if constexpr (sizeof(T) == 2 && bwd_filter_dot2_lds_bytes<D, KS>() <= kMaxLdsBytes) {
        return h->half16 ? bwd_filter_dot2<F16Fmt, D, KS>(h, launch, v, g, lds, s)
                         : bwd_filter_dot2<Bf16Fmt, D, KS>(h, launch, v, g, lds, s);
    } else if constexpr (bytes > kMaxLdsBytes) {
        // more LDS than a compute unit has: create refuses the shape, no kernel is built for it
        if (bytes > *lds) *lds = bytes;
        return launch ? hipErrorInvalidValue : hipSuccess;
    } else {
        if (!launch) {
            if (bytes > *lds) *lds = bytes;
            return hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_filter_kernel<T, D, KS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(bytes));
        }
        const T *vg, *gg;
        const BwdFilterParams p = bwd_filter_params<T>(h, kApplyTH, v, g, &vg, &gg);
        hipLaunchKernelGGL((bwd_filter_kernel<T, D, KS>), dim3(h->filter_chunks, h->units),
                           dim3(kBwdFilterThreads), bytes, s, vg, gg, h->fpart, h->desc.heads, p);
        return hipGetLastError();
    }
}

template <typename T, int D>
hipError_t bwd_filter(castling_attn* h, bool launch, const void* v, const void* g, size_t* lds,
                      hipStream_t s)
{
    switch (h->desc.dw_kernel) {
        case 1: return bwd_filter_ks<T, D, 1>(h, launch, v, g, lds, s);
        case 3: return bwd_filter_ks<T, D, 3>(h, launch, v, g, lds, s);
        case 5: return bwd_filter_ks<T, D, 5>(h, launch, v, g, lds, s);
        case 7: return bwd_filter_ks<T, D, 7>(h, launch, v, g, lds, s);
        default: return bwd_filter_ks<T, D, 9>(h, launch, v, g, lds, s);
    }
}

// ------------------------------------------------------------------ one-kernel path
template <int KS, bool LIN, bool DW, typename X>
hipError_t fused_branches(castling_attn* h, bool launch, const void* q, const void* k,
                          const void* v, const void* w, const void* bias, void* out, hipStream_t s)
{
    // only the linear branch tells a pair of heads from one head
    constexpr bool kPairKernel = LIN;
    const bool pair = kPairKernel && h->pair;
    if (!launch) {
        const void* fn = reinterpret_cast<const void*>(&fused_small_kernel<KS, LIN, DW, X, false>);
        if constexpr (kPairKernel)
            if (pair) fn = reinterpret_cast<const void*>(&fused_small_kernel<KS, LIN, DW, X, true>);
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLdsBytes);
    }
    const castling_attn_desc_t& d = h->desc;
    FusedParams p = {};
    p.N = d.N;
    p.grid_h = d.grid_h;
    p.grid_w = d.grid_w;
    p.extra = d.extra_tokens;
    p.norm_none = d.norm == CASTLING_NORM_NONE;
    p.eps = d.eps;
    p.in = h->apply_in;
    p.out = h->apply_out;
    p.in_skew = h->in_skew;
    p.out_skew = h->out_skew;
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(h->apply_units), dim3(256), kFusedLdsBytes, s,
                           static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                           static_cast<const bf16_t*>(v), static_cast<const bf16_t*>(w),
                           static_cast<const bf16_t*>(bias),
                           (d.flags & CASTLING_FLAG_KEEP_STATE) ? h->state : nullptr,
                           static_cast<bf16_t*>(out), h->apply_heads, p);
    };
    if constexpr (kPairKernel) {
        if (pair) go(fused_small_kernel<KS, LIN, DW, X, true>);
        else go(fused_small_kernel<KS, LIN, DW, X, false>);
    } else {
        go(fused_small_kernel<KS, LIN, DW, X, false>);
    }
    h->state_valid = (d.flags & CASTLING_FLAG_KEEP_STATE) != 0;
    h->apply_ready = false;  // the operand tables stayed on chip
    return hipGetLastError();
}

template <int KS, typename X>
hipError_t fused_fmt(castling_attn* h, bool launch, const void* q, const void* k, const void* v,
                     const void* w, const void* bias, void* out, hipStream_t s)
{
    const bool lin = (h->desc.branches & CASTLING_BRANCH_LINEAR) != 0;
    const bool dw = (h->desc.branches & CASTLING_BRANCH_DWCONV) != 0;
    if (lin && dw) return fused_branches<KS, true, true, X>(h, launch, q, k, v, w, bias, out, s);
    if (lin) return fused_branches<KS, true, false, X>(h, launch, q, k, v, w, bias, out, s);
    return fused_branches<KS, false, true, X>(h, launch, q, k, v, w, bias, out, s);
}

template <int KS>
hipError_t fused_ks(castling_attn* h, bool launch, const void* q, const void* k, const void* v,
                    const void* w, const void* bias, void* out, hipStream_t s)
{
    return h->half16 ? fused_fmt<KS, F16Fmt>(h, launch, q, k, v, w, bias, out, s)
                     : fused_fmt<KS, Bf16Fmt>(h, launch, q, k, v, w, bias, out, s);
}

hipError_t do_fused(castling_attn* h, bool launch, const void* q, const void* k, const void* v,
                    const void* w, const void* bias, void* out, hipStream_t s)
{
    switch (h->desc.dw_kernel) {
        case 1: return fused_ks<1>(h, launch, q, k, v, w, bias, out, s);
        case 3: return fused_ks<3>(h, launch, q, k, v, w, bias, out, s);
        default: return fused_ks<5>(h, launch, q, k, v, w, bias, out, s);
    }
}


bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

bool overlaps(const void* a, size_t a_bytes, const void* b, size_t b_bytes)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

int check_apply_args(castling_attn_t h, const void* q, const void* v, const void* dw_weight,
                     void* out)
{
    if (!h || !out) return CASTLING_ERR_INVALID_ARG;
    const castling_attn_desc_t& d = h->desc;
    const bool lin = d.branches & CASTLING_BRANCH_LINEAR, dw = d.branches & CASTLING_BRANCH_DWCONV;
    if ((lin && !q) || (dw && (!v || !dw_weight))) return CASTLING_ERR_INVALID_ARG;
    if (misaligned(out) || (lin && misaligned(q)) || (dw && (misaligned(v) || misaligned(dw_weight))))
        return CASTLING_ERR_INVALID_ARG;
    if ((lin && overlaps(out, h->out_span, q, h->q_span)) ||
        (dw && overlaps(out, h->out_span, v, h->in_span)))
        return CASTLING_ERR_ALIAS;
    return CASTLING_OK;
}

// Everything castling_attn_create decides before it allocates: kernel paths, token split, launch
// attributes, and the sizes of the workspace parts (h->parts, h->workspace_bytes).  desc has
// passed castling_attn_validate.  No pointer into the workspace is set here.
int plan_handle(const castling_attn_desc_t* desc, castling_attn* h)
{
    h->desc = *desc;
    if (h->desc.branches == 0) h->desc.branches = CASTLING_BRANCH_ALL;
    if (h->desc.eps == 0.0f) h->desc.eps = 1e-12f;
    h->units = desc->B * desc->heads;
    h->state_valid = false;
    h->apply_ready = false;
    {
        const castling_attn_desc_t& d = h->desc;
        h->pool = d.q_pool == 2 ? 2 : 1;
        h->qgrid_h = (d.grid_h + h->pool - 1) / h->pool;
        h->qgrid_w = (d.grid_w + h->pool - 1) / h->pool;
        h->nq = h->pool == 1 ? d.N : h->qgrid_h * h->qgrid_w;
        h->residual_q = (d.flags & CASTLING_FLAG_RESIDUAL_Q) != 0;
        auto dense = [&](int n) {
            return TensorStrides{static_cast<long long>(d.heads) * n * d.d,
                                 static_cast<long long>(n) * d.d, d.d};
        };
        h->in_st = d.in_stride_n ? TensorStrides{d.in_stride_b, d.in_stride_h, d.in_stride_n}
                                 : dense(d.N);
        h->out_st = d.out_stride_n ? TensorStrides{d.out_stride_b, d.out_stride_h, d.out_stride_n}
                                   : dense(h->nq);
        h->q_st = h->pool == 1 ? h->in_st
                  : d.q_stride_n ? TensorStrides{d.q_stride_b, d.q_stride_h, d.q_stride_n}
                                 : dense(h->nq);
        auto span = [&](const TensorStrides& s, int n) {
            return static_cast<size_t>((d.B - 1) * s.b + (d.heads - 1) * s.h + (n - 1) * s.n + d.d) *
                   dtype_size(d.io_dtype);
        };
        h->in_span = span(h->in_st, d.N);
        h->out_span = span(h->out_st, h->nq);
        h->q_span = span(h->q_st, h->nq);
    }
    h->dpad = desc->d <= 16 ? 16 : desc->d <= 32 ? 32 : desc->d <= 64 ? 64 : 128;
    h->state_size = h->dpad * h->dpad + 2 * h->dpad;

    const bool allow_mfma = (desc->io_dtype == CASTLING_BF16 || desc->io_dtype == CASTLING_F16) &&
                            !(desc->flags & CASTLING_FLAG_VECTOR_ALU);
    h->half16 = desc->io_dtype == CASTLING_F16;
    h->mfma_reduce = allow_mfma && (desc->d == 32 || desc->d == 64);
    // pooled or residual queries: pass 2 on the vector-ALU kernel (pass 1 is the same work)
    const bool plain_q = h->pool == 1 && !h->residual_q;
    h->mfma_apply = allow_mfma && desc->d == 64 && plain_q;
    h->apply_units = h->units;
    h->apply_heads = desc->heads;
    h->apply_in = h->in_st;
    h->apply_out = h->out_st;
    h->in_skew = h->out_skew = 0;
    h->pair = h->pair_reduce = false;
    if (allow_mfma && desc->d == 32 && desc->heads % 2 == 0 && plain_q) {
        // two neighbouring heads of 32 channels as one unit of 64 for pass 2: the second half of
        // a token row lies one head stride further on instead of 64 bytes
        const long long in_skew = h->in_st.h * 2 - 64, out_skew = h->out_st.h * 2 - 64;
        const long long lim = (1ll << 32) - 256;
        if (in_skew >= 0 && out_skew >= 0 && desc->N * h->in_st.n * 2 + in_skew < lim &&
            desc->N * h->out_st.n * 2 + out_skew < lim) {
            h->pair = h->mfma_apply = true;
            h->apply_units = h->units / 2;
            h->apply_heads = desc->heads / 2;
            h->apply_in.h *= 2;
            h->apply_out.h *= 2;
            h->in_skew = static_cast<uint32_t>(in_skew);
            h->out_skew = static_cast<uint32_t>(out_skew);
            // pass 1 gains from pairs only where they make its loads whole 128-byte rows
            h->pair_reduce = in_skew == 0;
        }
    }
    const bool separate = (desc->flags & CASTLING_FLAG_SEPARATE_PASSES) != 0;
    h->fused = h->mfma_apply && desc->N <= kFusedMaxTokens && desc->dw_kernel <= kFusedMaxKs && !separate;
    // token split: enough blocks to fill the chip; chunks a multiple of what one block
    // stages per iteration (128 tokens for the MFMA kernel, at most 64 for the generic one)
    const int target_blocks = kTargetReduceBlocks;
    const int reduce_units = h->pair_reduce ? h->apply_units : h->units;
    int n_split = target_blocks / reduce_units;  // never one block more than fits at once
    const int max_split = (desc->N + kMinChunkTokens - 1) / kMinChunkTokens;
    if (n_split > max_split) n_split = max_split;
    if (n_split < 1) n_split = 1;
    int chunk = (desc->N + n_split - 1) / n_split;
    const int chunk_mult = kReduceWaves * kReduceIterTokens;
    chunk = ((chunk + chunk_mult - 1) / chunk_mult) * chunk_mult;
    h->chunk = chunk;
    h->n_split = (desc->N + chunk - 1) / chunk;

    hipError_t e = hipGetDevice(&h->device);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&h->num_cus, hipDeviceAttributeMultiprocessorCount, h->device);
    if (e == hipSuccess && h->num_cus < 1) h->num_cus = 1;
    if (e == hipSuccess) e = do_apply(h, false, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    if (e == hipSuccess && h->fused)
        e = do_fused(h, false, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    if (e == hipSuccess) {
        int max_lds = 0;
        e = hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, h->device);
        if (e == hipSuccess && h->apply_lds > static_cast<size_t>(max_lds)) {
            return CASTLING_ERR_UNSUPPORTED;
        }
    }
    // backward pass: LDS attributes of its kernels, and of the vector-ALU pass 2 it may need
    h->training = (desc->flags & CASTLING_FLAG_TRAINING) != 0;
    h->ov.on = h->ov.generic = false;
    WorkspaceParts& ws = h->parts;
    ws = WorkspaceParts{};
    // CASTLING_FLAG_VECTOR_ALU keeps the per-row kernels of the backward off the matrix cores too
    h->mfma_rows = allow_mfma && (desc->d == 32 || desc->d == 64);
    if (e == hipSuccess && h->training) {
        size_t lds = 0;
        const size_t keep = h->apply_lds;
        h->ov.on = h->ov.generic = true;
        h->ov.q = h->ov.v = h->ov.out = h->in_st;
        h->ov.lin_scale = 1.0f;
        e = do_apply(h, false, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
        lds = h->apply_lds;
        h->apply_lds = keep;
        h->ov.on = h->ov.generic = false;
        if (e == hipSuccess)
            e = dispatch_type_width(desc->io_dtype, h->dpad, [&](auto t, auto dc) {
                using T = decltype(t);
                constexpr int D = decltype(dc)::value;
                hipError_t r = bwd_rows<T, D>(h, false, true, nullptr, nullptr, nullptr, &lds, nullptr);
                if (r == hipSuccess) r = bwd_filter<T, D>(h, false, nullptr, nullptr, &lds, nullptr);
                return r;
            });
        if (e == hipSuccess && lds > kMaxLdsBytes) {
            return CASTLING_ERR_UNSUPPORTED;
        }
        const int taps1 = desc->dw_kernel * desc->dw_kernel + 1;
        const int n_tiles = ((desc->grid_w + kApplyTW - 1) / kApplyTW) *
                            ((desc->grid_h + kApplyTH - 1) / kApplyTH);
        h->row_tiles = (desc->N + kBwdTokens - 1) / kBwdTokens;
        h->qrow_tiles = (h->nq + kBwdTokens - 1) / kBwdTokens;
        h->kb_parts = h->mfma_rows ? 4 * h->qrow_tiles : h->qrow_tiles;
        h->filter_chunks = std::max(1, std::min(n_tiles, 1024 / h->units));
        ws.a = align_up(h->in_span, 256) * (h->pool == 2 ? 3 : 1);  // a; pooled: + q_up, g_up
        ws.kbp = align_up(sizeof(float) * static_cast<size_t>(h->units) * h->kb_parts * h->dpad, 256);
        ws.kb = align_up(sizeof(float) * static_cast<size_t>(h->units) * h->dpad, 256);
        ws.wflip = align_up(dtype_size(desc->io_dtype) * static_cast<size_t>(desc->heads) * desc->d *
                                   (taps1 - 1), 256);
        ws.fpart = align_up(sizeof(float) * static_cast<size_t>(h->units) * h->filter_chunks * taps1 *
                                   h->dpad, 256);
    }
    // one block of memory, 256-byte aligned parts
    ws.partial =
        h->pair_reduce ? align_up(sizeof(float) * static_cast<size_t>(h->apply_units) * h->n_split *
                               StateLayout<64>::SIZE, 256)
                : align_up(sizeof(float) * static_cast<size_t>(h->units) * h->n_split * h->state_size, 256);
    ws.state =
        align_up(sizeof(float) * static_cast<size_t>(h->units) * h->state_size, 256);
    if (h->mfma_apply) {
        ws.sfrag = align_up(sizeof(bf16_t) * static_cast<size_t>(h->units) * kSfragPerUnit, 256);
        ws.kfrag = align_up(sizeof(bf16_t) * static_cast<size_t>(h->units) * kKfragPerUnit, 256);
        ws.vhalf = align_up(sizeof(float) * static_cast<size_t>(h->units) * 64, 256);
        ws.wfrag =
            align_up(static_cast<size_t>(desc->heads) * 4 * desc->dw_kernel * 3 * 64 * 8, 256);
    }
    h->workspace_bytes = ws.partial + ws.state + ws.sfrag + ws.kfrag + ws.vhalf + 2 * ws.wfrag + ws.a +
                         ws.kbp + ws.kb + ws.wflip + ws.fpart;
    if (e != hipSuccess) return hip_fail(e);
    // Small vector-ALU problems: every apply block sums the few partial states itself instead of
    // waiting for a combine launch (cfg1: three launches become two).  Not when the caller wants
    // the state kept, and not where many blocks would each re-read many partials.
    {
        const long long tiles = static_cast<long long>((desc->grid_w + kApplyTW - 1) / kApplyTW) *
                                ((desc->grid_h + kApplyTH - 1) / kApplyTH);
        h->sum_in_apply = !h->mfma_apply && h->n_split > 1 && h->n_split <= 4 && tiles <= 16 &&
                          !(desc->flags & CASTLING_FLAG_KEEP_STATE);
    }
    h->partials_pending = false;

    h->workspace = nullptr;
    return CASTLING_OK;
}

// Points the handle's parts into the block at base (h->workspace_bytes long, 256-byte aligned).
void carve_workspace(castling_attn* h, unsigned char* base)
{
    const WorkspaceParts& ws = h->parts;
    unsigned char* p = base;
    h->partial = reinterpret_cast<float*>(p);
    p += ws.partial;
    h->state = reinterpret_cast<float*>(p);
    p += ws.state;
    h->sfrag = reinterpret_cast<bf16_t*>(p);
    p += ws.sfrag;
    h->kfrag = reinterpret_cast<bf16_t*>(p);
    p += ws.kfrag;
    h->vhalf = reinterpret_cast<float*>(p);
    p += ws.vhalf;
    h->wfrag = reinterpret_cast<bf16_t*>(p);
    p += ws.wfrag;
    h->wfrag_reg = reinterpret_cast<bf16_t*>(p);
    p += ws.wfrag;
    h->a_buf = p;
    h->q_up = h->g_up = nullptr;
    if (h->training && h->pool == 2) {
        h->q_up = p + ws.a / 3;
        h->g_up = p + 2 * (ws.a / 3);
    }
    p += ws.a;
    h->kb_part = reinterpret_cast<float*>(p);
    p += ws.kbp;
    h->kb = reinterpret_cast<float*>(p);
    p += ws.kb;
    h->wflip = p;
    p += ws.wflip;
    h->fpart = reinterpret_cast<float*>(p);
    if (!h->mfma_apply && h->n_split == 1) h->partial = h->state;  // see do_reduce
}

// ------------------------------------------------------------------ scratch without allocation
// Workspace of castling_attn_forward_static.  The name is a host-side stand-in for the symbol:
// host code uses the per-device address from hipGetSymbolAddress, never the name itself.
constexpr size_t kStaticScratchBytes = CASTLING_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_base[kMaxDevices];  // per device: where its copy of `scratch` lies
bool g_static_plan_valid = false;
castling_attn_desc_t g_static_desc;
castling_attn g_static_plan;

// The address of the current device's copy of the array (looked up once per device).
hipError_t static_scratch_base(int device, unsigned char** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_base[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return hipErrorInvalidSymbol;
        g_static_base[device] = static_cast<unsigned char*>(p);
    }
    *out = g_static_base[device];
    return hipSuccess;
}

int forward_impl(castling_attn* h, const void* q, const void* k, const void* v,
                          const void* dw_weight, const void* dw_bias, void* out, void* stream)
{
    if (!h) return CASTLING_ERR_INVALID_ARG;
    // dw_weight == NULL: the filters registered by castling_attn_prepare_weights
    const bool registered = !dw_weight && h->prepared_w;
    const void* w = registered ? h->prepared_w : dw_weight;
    // every argument is checked before anything is enqueued
    int st = check_apply_args(h, q, v, w, out);
    if (st != CASTLING_OK) return st;
    const castling_attn_desc_t& d = h->desc;
    const size_t es = dtype_size(d.io_dtype);
    if ((d.branches & CASTLING_BRANCH_DWCONV) &&
        (overlaps(out, h->out_span, w, static_cast<size_t>(d.heads) * d.d * d.dw_kernel * d.dw_kernel * es) ||
         (dw_bias && overlaps(out, h->out_span, dw_bias, static_cast<size_t>(d.heads) * d.d * es))))
        return CASTLING_ERR_ALIAS;
    if (d.branches & CASTLING_BRANCH_LINEAR) {
        if (!k || !v || misaligned(k) || misaligned(v)) return CASTLING_ERR_INVALID_ARG;
        if (overlaps(out, h->out_span, k, h->in_span) || overlaps(out, h->out_span, v, h->in_span))
            return CASTLING_ERR_ALIAS;
    }
    if (d.branches & CASTLING_BRANCH_LINEAR) {
        if (h->fused) {
            HIP_TRY(do_fused(h, true, q, k, v, w, dw_bias, out, static_cast<hipStream_t>(stream)));
            return CASTLING_OK;
        }
        // the combine launch also prepares the weight operands of the MFMA apply kernel, unless
        // the registered filters' table is the one to use
        const bool fuse_w = h->mfma_apply && (d.branches & CASTLING_BRANCH_DWCONV);
        st = do_reduce(h, k, v, fuse_w && !registered ? w : nullptr, static_cast<hipStream_t>(stream),
                       h->sum_in_apply);
        if (st != CASTLING_OK) return st;
        if (fuse_w) {
            h->use_registered = registered;
            const hipError_t e = do_apply(h, true, q, v, nullptr, dw_bias, out, static_cast<hipStream_t>(stream));
            h->use_registered = false;
            HIP_TRY(e);
            return CASTLING_OK;
        }
    }
    if (h->fused) {  // convolution branch alone
        HIP_TRY(do_fused(h, true, q, k, v, w, dw_bias, out, static_cast<hipStream_t>(stream)));
        return CASTLING_OK;
    }
    return castling_attn_apply(h, q, v, dw_weight, dw_bias, out, stream);
}

}  // namespace

extern "C" {

const char* castling_attn_strerror(int status)
{
    switch (status) {
        case CASTLING_OK: return "ok";
        case CASTLING_ERR_INVALID_ARG: return "invalid argument";
        case CASTLING_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case CASTLING_ERR_HIP: return g_hip_error;
        case CASTLING_ERR_ALIAS: return "an output overlaps an input or another output";
        case CASTLING_ERR_TOO_LARGE:
            return "the problem needs more scratch memory than castling_attn_forward_static holds "
                   "(CASTLING_STATIC_SCRATCH_BYTES); use a handle";
        default: return "unknown status";
    }
}

int castling_attn_validate(const castling_attn_desc_t* d)
{
    if (!d) return CASTLING_ERR_INVALID_ARG;
    if (d->B <= 0 || d->heads <= 0 || d->N <= 0 || d->d <= 0 || d->grid_h <= 0 || d->grid_w <= 0 ||
        d->dw_kernel <= 0)
        return CASTLING_ERR_INVALID_ARG;
    if (d->extra_tokens < 0 || d->extra_tokens > 64) return CASTLING_ERR_INVALID_ARG;
    if (static_cast<int64_t>(d->grid_h) * d->grid_w + d->extra_tokens != d->N)
        return CASTLING_ERR_INVALID_ARG;
    if (d->dw_kernel % 2 == 0) return CASTLING_ERR_INVALID_ARG;
    if (d->norm != CASTLING_NORM_ROWSUM && d->norm != CASTLING_NORM_NONE)
        return CASTLING_ERR_INVALID_ARG;
    if (d->branches & ~static_cast<uint32_t>(CASTLING_BRANCH_ALL)) return CASTLING_ERR_INVALID_ARG;
    // the kernels form 1 / eps: a floor below the smallest normal float would make it infinite
    if (!(d->eps >= 0.0f) || (d->eps > 0.0f && d->eps < FLT_MIN)) return CASTLING_ERR_INVALID_ARG;
    if (d->flags & ~static_cast<uint32_t>(CASTLING_FLAG_KEEP_STATE | CASTLING_FLAG_RESIDUAL_Q |
                                          CASTLING_FLAG_TRAINING | CASTLING_FLAG_SEPARATE_PASSES |
                                          CASTLING_FLAG_VECTOR_ALU))
        return CASTLING_ERR_INVALID_ARG;
    if (d->io_dtype != CASTLING_F32 && d->io_dtype != CASTLING_BF16 && d->io_dtype != CASTLING_F16)
        return CASTLING_ERR_UNSUPPORTED;
    if (d->d % 8 != 0 || d->d > 128) return CASTLING_ERR_UNSUPPORTED;
    if (d->dw_kernel > 9) return CASTLING_ERR_UNSUPPORTED;
    // grid.y carries the unit index; keep element offsets inside int64 comfortably
    if (static_cast<int64_t>(d->B) * d->heads > 65535) return CASTLING_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(d->B) * d->heads * d->N * d->d > (int64_t(1) << 40))
        return CASTLING_ERR_UNSUPPORTED;
    if (d->q_pool < 0 || d->reserved0 != 0) return CASTLING_ERR_INVALID_ARG;
    if (d->q_pool > 2 || (d->q_pool == 2 && d->extra_tokens != 0)) return CASTLING_ERR_UNSUPPORTED;
    if (d->q_pool != 2 && (d->q_stride_b != 0 || d->q_stride_h != 0 || d->q_stride_n != 0))
        return CASTLING_ERR_INVALID_ARG;
    if ((d->flags & CASTLING_FLAG_RESIDUAL_Q) && d->branches != 0 &&
        !(d->branches & CASTLING_BRANCH_LINEAR))
        return CASTLING_ERR_INVALID_ARG;
    const int64_t es = static_cast<int64_t>(dtype_size(d->io_dtype));
    const int64_t sets[3][3] = {{d->in_stride_b, d->in_stride_h, d->in_stride_n},
                                {d->out_stride_b, d->out_stride_h, d->out_stride_n},
                                {d->q_stride_b, d->q_stride_h, d->q_stride_n}};
    for (const auto& s : sets) {
        const bool dense = s[0] == 0 && s[1] == 0 && s[2] == 0;  // contiguous default
        if (!dense) {
            for (int i = 0; i < 3; ++i)
                if (s[i] <= 0 || (s[i] * es) % 16 != 0) return CASTLING_ERR_INVALID_ARG;
            if (s[2] < d->d) return CASTLING_ERR_INVALID_ARG;
            if (s[0] > (int64_t(1) << 40) || s[1] > (int64_t(1) << 40))
                return CASTLING_ERR_UNSUPPORTED;
        }
        // the kernels address tokens of one unit with 32-bit byte offsets
        const int64_t tok = dense ? d->d : s[2];
        if (tok > (int64_t(1) << 32) || d->N * tok * es >= (int64_t(1) << 32))
            return CASTLING_ERR_UNSUPPORTED;
    }
    // pass 2 counts its work items (4 rows x 16 columns of one unit) in 32 bits
    const int64_t steps = static_cast<int64_t>(d->B) * d->heads * ((d->grid_w + 15) / 16) *
                          ((d->grid_h + 3) / 4);
    if (steps > (int64_t(1) << 30)) return CASTLING_ERR_UNSUPPORTED;
    return CASTLING_OK;
}

int castling_attn_create(const castling_attn_desc_t* desc, castling_attn_t* out_handle)
{
    if (!out_handle) return CASTLING_ERR_INVALID_ARG;
    *out_handle = nullptr;
    int st = castling_attn_validate(desc);
    if (st != CASTLING_OK) return st;

    castling_attn* h = new (std::nothrow) castling_attn();
    if (!h) return hip_fail(hipErrorOutOfMemory);
    st = plan_handle(desc, h);
    if (st != CASTLING_OK) {
        delete h;
        return st;
    }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&h->workspace), h->workspace_bytes);
    if (e != hipSuccess) {
        delete h;
        return hip_fail(e);
    }
    carve_workspace(h, h->workspace);
    if (h->training && h->pool == 2) {
        // a, q_up, g_up hold rows only where pooled queries stand; the rest stays zero for good
        e = hipMemset(h->a_buf, 0, h->parts.a);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);  // before any stream's kernels
        if (e != hipSuccess) {
            (void)hipFree(h->workspace);
            delete h;
            return hip_fail(e);
        }
    }
    *out_handle = h;
    return CASTLING_OK;
}

int castling_attn_destroy(castling_attn_t h)
{
    if (!h) return CASTLING_OK;
    hipError_t e = h->workspace ? hipFree(h->workspace) : hipSuccess;
    delete h;
    return e == hipSuccess ? CASTLING_OK : hip_fail(e);
}

size_t castling_attn_workspace_bytes(castling_attn_t h) { return h ? h->workspace_bytes : 0; }

int castling_attn_num_splits(castling_attn_t h) { return h ? h->n_split : 0; }

int castling_attn_num_launches(castling_attn_t h)
{
    if (!h) return 0;
    const bool lin = (h->desc.branches & CASTLING_BRANCH_LINEAR) != 0;
    const int extra = h->desc.extra_tokens > 0 ? 1 : 0;  // the tokens off the grid: one more launch
    if (h->fused) return 1;
    if (!lin) return 1 + extra;
    return ((h->n_split == 1 && !h->pair) || h->sum_in_apply ? 2 : 3) + extra;
}

int castling_attn_reduce(castling_attn_t h, const void* k, const void* v, void* stream)
{
    if (!h || !k || !v) return CASTLING_ERR_INVALID_ARG;
    if (misaligned(k) || misaligned(v)) return CASTLING_ERR_INVALID_ARG;
    return do_reduce(h, k, v, nullptr, static_cast<hipStream_t>(stream));
}

int castling_attn_prepare_weights(castling_attn_t h, const void* dw_weight, void* stream)
{
    if (!h || !dw_weight || misaligned(dw_weight)) return CASTLING_ERR_INVALID_ARG;
    if (h->mfma_apply && (h->desc.branches & CASTLING_BRANCH_DWCONV)) {
        const castling_attn_desc_t& d = h->desc;
        const int threads = h->apply_heads * 4 * d.dw_kernel * 3 * 64;
        hipLaunchKernelGGL(dwconv_weight_frag_kernel, dim3((threads + 255) / 256), dim3(256), 0,
                           static_cast<hipStream_t>(stream), static_cast<const bf16_t*>(dw_weight),
                           h->wfrag_reg, h->apply_heads, d.dw_kernel);
        HIP_TRY(hipGetLastError());
    }
    h->prepared_w = dw_weight;
    return CASTLING_OK;
}

int castling_attn_apply(castling_attn_t h, const void* q, const void* v, const void* dw_weight,
                        const void* dw_bias, void* out, void* stream)
{
    if (!h) return CASTLING_ERR_INVALID_ARG;
    const bool registered = !dw_weight && h->prepared_w;
    const void* w = registered ? h->prepared_w : dw_weight;
    int st = check_apply_args(h, q, v, w, out);
    if (st != CASTLING_OK) return st;
    if ((h->desc.branches & CASTLING_BRANCH_LINEAR) && !h->apply_ready)
        return CASTLING_ERR_INVALID_ARG;  // no reduce has left a state to apply
    // the matrix-core path already holds the registered filters in an operand table of their own
    h->use_registered = registered && h->mfma_apply;
    const hipError_t e = do_apply(h, true, q, v, h->use_registered ? nullptr : w, dw_bias, out,
                                  static_cast<hipStream_t>(stream));
    h->use_registered = false;
    HIP_TRY(e);
    return CASTLING_OK;
}

int castling_attn_pairwise(castling_attn_t h, const castling_pair_params_t* params, const void* q,
                           const void* k, const void* v, void* out, uint64_t* kept, void* stream)
{
    if (!h || !params || !q || !k || !v || !out) return CASTLING_ERR_INVALID_ARG;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out))
        return CASTLING_ERR_INVALID_ARG;
    if (params->mode != CASTLING_PAIR_SPARSE_SOFTMAX && params->mode != CASTLING_PAIR_ANGULAR)
        return CASTLING_ERR_INVALID_ARG;
    if (params->accumulate & ~1) return CASTLING_ERR_INVALID_ARG;
    const bool sparse = params->mode == CASTLING_PAIR_SPARSE_SOFTMAX;
    if (sparse && (!(params->threshold >= 0.0f) || !(params->threshold <= 1.0f) ||
                   !(params->scale == params->scale) || (params->normalize & ~1)))
        return CASTLING_ERR_INVALID_ARG;
    if (kept && (reinterpret_cast<uintptr_t>(kept) & 7u)) return CASTLING_ERR_INVALID_ARG;
    if (overlaps(out, h->out_span, q, h->q_span) || overlaps(out, h->out_span, k, h->in_span) ||
        overlaps(out, h->out_span, v, h->in_span))
        return CASTLING_ERR_ALIAS;
    const castling_attn_desc_t& d = h->desc;
    const bool half = d.io_dtype == CASTLING_F16;
    if ((d.io_dtype != CASTLING_BF16 && !half) || d.d != 64 || h->pool != 1)
        return CASTLING_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    PairParams p = {};
    p.N = d.N;
    p.normalize = params->normalize;
    p.accumulate = params->accumulate;
    p.norm_none = d.norm == CASTLING_NORM_NONE;
    p.scale = params->scale;
    p.threshold = params->threshold;
    p.eps = d.eps;
    p.in = h->in_st;
    p.out = h->out_st;
    unsigned long long* cnt = reinterpret_cast<unsigned long long*>(kept);
    if (sparse && cnt) {
        // counters start at zero; a fill kernel, so that the call can be captured in a graph
        hipLaunchKernelGGL(zero_u64_kernel, dim3((h->units + 255) / 256), dim3(256), 0, s, cnt,
                           h->units);
        HIP_TRY(hipGetLastError());
    }
    const dim3 grid((d.N + 127) / 128, h->units), block(256);
    const bf16_t* q16 = static_cast<const bf16_t*>(q);
    const bf16_t* k16 = static_cast<const bf16_t*>(k);
    const bf16_t* v16 = static_cast<const bf16_t*>(v);
    bf16_t* o16 = static_cast<bf16_t*>(out);
    if (sparse) {
        if (half)
            hipLaunchKernelGGL((pairwise_attn_kernel<kPairSparse, F16Fmt>), grid, block, 0, s, q16,
                               k16, v16, o16, cnt, d.heads, p);
        else
            hipLaunchKernelGGL((pairwise_attn_kernel<kPairSparse, Bf16Fmt>), grid, block, 0, s, q16,
                               k16, v16, o16, cnt, d.heads, p);
    } else {
        if (half)
            hipLaunchKernelGGL((pairwise_attn_kernel<kPairAngular, F16Fmt>), grid, block, 0, s, q16,
                               k16, v16, o16, nullptr, d.heads, p);
        else
            hipLaunchKernelGGL((pairwise_attn_kernel<kPairAngular, Bf16Fmt>), grid, block, 0, s,
                               q16, k16, v16, o16, nullptr, d.heads, p);
    }
    HIP_TRY(hipGetLastError());
    return CASTLING_OK;
}

int castling_attn_forward(castling_attn_t h, const void* q, const void* k, const void* v,
                          const void* dw_weight, const void* dw_bias, void* out, void* stream)
{
    return forward_impl(h, q, k, v, dw_weight, dw_bias, out, stream);
}

int castling_attn_forward_static(const castling_attn_desc_t* desc, const void* q, const void* k,
                                 const void* v, const void* dw_weight, const void* dw_bias, void* out,
                                 void* stream)
{
    int st = castling_attn_validate(desc);
    if (st != CASTLING_OK) return st;
    if (desc->flags & CASTLING_FLAG_TRAINING) return CASTLING_ERR_INVALID_ARG;  // no backward here
    int device = -1;
    HIP_TRY(hipGetDevice(&device));
    // the plan of the last descriptor seen on this device is kept: a repeated call makes no
    // HIP call besides its launches
    castling_attn h{};
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (g_static_plan_valid && g_static_plan.device == device &&
            std::memcmp(&g_static_desc, desc, sizeof(*desc)) == 0) {
            h = g_static_plan;
        } else {
            g_static_plan_valid = false;
            st = plan_handle(desc, &h);
            if (st != CASTLING_OK) return st;
            g_static_plan = h;
            std::memcpy(&g_static_desc, desc, sizeof(*desc));
            g_static_plan_valid = true;
        }
    }
    if (h.workspace_bytes > kStaticScratchBytes) return CASTLING_ERR_TOO_LARGE;
    unsigned char* base = nullptr;
    HIP_TRY(static_scratch_base(device, &base));
    carve_workspace(&h, base);
    return forward_impl(&h, q, k, v, dw_weight, dw_bias, out, stream);
}

int castling_attn_backward(castling_attn_t h, const void* q, const void* k, const void* v,
                           const void* dw_weight, const void* grad_out, void* grad_q, void* grad_k,
                           void* grad_v, float* grad_w, float* grad_bias, void* stream)
{
    if (!h || !h->training) return CASTLING_ERR_INVALID_ARG;
    const castling_attn_desc_t& d = h->desc;
    const bool lin = (d.branches & CASTLING_BRANCH_LINEAR) != 0;
    const bool dw = (d.branches & CASTLING_BRANCH_DWCONV) != 0;
    if (!q || !k || !v || !grad_out || !grad_q || !grad_k || !grad_v || (dw && (!dw_weight || !grad_w)))
        return CASTLING_ERR_INVALID_ARG;
    const void* ptrs[] = {q, k, v, grad_out, grad_q, grad_k, grad_v, dw ? dw_weight : nullptr};
    for (const void* ptr : ptrs)
        if (misaligned(ptr)) return CASTLING_ERR_INVALID_ARG;
    // no gradient may overlap an input or another gradient
    const void* ins[] = {q, k, v, grad_out};
    const size_t in_bytes[] = {h->q_span, h->in_span, h->in_span, h->out_span};
    void* outs[] = {grad_q, grad_k, grad_v};
    const size_t out_bytes[] = {h->q_span, h->in_span, h->in_span};
    for (int o = 0; o < 3; ++o) {
        for (int i = 0; i < 4; ++i)
            if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return CASTLING_ERR_ALIAS;
        for (int o2 = o + 1; o2 < 3; ++o2)
            if (outs[o] == outs[o2]) return CASTLING_ERR_ALIAS;
    }
    // ... the fp32 filter and bias gradients included, and no gradient may overlap the filters
    const size_t w_elems = static_cast<size_t>(d.heads) * d.d * d.dw_kernel * d.dw_kernel;
    const size_t b_elems = static_cast<size_t>(d.heads) * d.d;
    const size_t es = dtype_size(d.io_dtype);
    const void* fouts[] = {grad_w, grad_bias};
    const size_t fout_bytes[] = {w_elems * sizeof(float), b_elems * sizeof(float)};
    for (int f = 0; f < 2; ++f) {
        if (!fouts[f]) continue;
        for (int i = 0; i < 4; ++i)
            if (overlaps(fouts[f], fout_bytes[f], ins[i], in_bytes[i])) return CASTLING_ERR_ALIAS;
        for (int o = 0; o < 3; ++o)
            if (overlaps(fouts[f], fout_bytes[f], outs[o], out_bytes[o])) return CASTLING_ERR_ALIAS;
        if (dw && overlaps(fouts[f], fout_bytes[f], dw_weight, w_elems * es)) return CASTLING_ERR_ALIAS;
    }
    if (grad_w && grad_bias && overlaps(grad_w, fout_bytes[0], grad_bias, fout_bytes[1]))
        return CASTLING_ERR_ALIAS;
    if (dw)
        for (int o = 0; o < 3; ++o)
            if (overlaps(outs[o], out_bytes[o], dw_weight, w_elems * es)) return CASTLING_ERR_ALIAS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int taps = d.dw_kernel * d.dw_kernel;
    // pooled queries: the query-side kernel puts q, a, g on their places in the fine grid (zero
    // elsewhere) and the later passes run on the grid of k and v as they are
    const bool pooled = h->pool == 2;
    h->state_valid = false;  // the workspace ends up holding the state of (q, a), not of (k, v)
    h->apply_ready = false;
    h->partials_pending = false;
    int st = CASTLING_OK;
    hipError_t e = hipSuccess;
    auto typed = [&](auto&& f) { return dispatch_type_width(d.io_dtype, h->dpad, f); };
    if (lin) {
        // forward state of (k, v); a, b, dq per query row; the state of (q, a); kb'
        st = do_reduce(h, k, v, nullptr, s);
        if (st != CASTLING_OK) return st;
        e = typed([&](auto t, auto dc) {
            return bwd_rows<decltype(t), decltype(dc)::value>(h, true, true, q, grad_out, grad_q,
                                                               nullptr, s);
        });
        HIP_TRY(e);
        hipLaunchKernelGGL(bwd_vec_combine_kernel, dim3(h->units), dim3(1024), 0, s, h->kb_part, h->kb,
                           h->kb_parts, h->dpad);
        HIP_TRY(hipGetLastError());
        st = do_reduce(h, pooled ? h->q_up : q, h->a_buf, nullptr, s);
        if (st != CASTLING_OK) return st;
        h->state_valid = false;
        // dk per key row from the state of (q, a)
        e = typed([&](auto t, auto dc) {
            return bwd_rows<decltype(t), decltype(dc)::value>(h, true, false, k, v, grad_k, nullptr, s);
        });
        HIP_TRY(e);
    } else {
        // no attention branch: q and k do not reach the output
        typed([&](auto t, auto) {
            using T = decltype(t);
            const int per_row = d.d / IO<T>::VEC;
            hipLaunchKernelGGL(zero_rows_kernel<T>, dim3((h->nq * per_row + 255) / 256, h->units),
                               dim3(256), 0, s, static_cast<T*>(grad_q), h->nq, d.d, d.heads, h->q_st);
            hipLaunchKernelGGL(zero_rows_kernel<T>, dim3((d.N * per_row + 255) / 256, h->units),
                               dim3(256), 0, s, static_cast<T*>(grad_k), d.N, d.d, d.heads, h->in_st);
            return 0;
        });
        HIP_TRY(hipGetLastError());
    }
    // dv: pass 2 on (k, g) with the state of (q, a), the filters turned by 180 degrees, no
    // normaliser, no bias; written in the layout of v
    if (dw) {
        const int n = d.heads * d.d * taps;
        typed([&](auto t, auto) {
            using T = decltype(t);
            hipLaunchKernelGGL(flip_filters_kernel<T>, dim3((n + 255) / 256), dim3(256), 0, s,
                               static_cast<const T*>(dw_weight), static_cast<T*>(h->wflip), n, taps);
            return 0;
        });
        HIP_TRY(hipGetLastError());
    }
    h->ov.on = true;
    h->ov.q = h->in_st;
    h->ov.v = pooled ? h->in_st : h->out_st;
    h->ov.out = h->in_st;
    h->ov.lin_scale = 1.0f / bwd_a_scale(h);
    h->ov.generic = h->ov.v.b != h->in_st.b || h->ov.v.h != h->in_st.h || h->ov.v.n != h->in_st.n;
    h->apply_ready = lin;
    const void* g_fine = grad_out;
    if (pooled) {
        g_fine = h->g_up;
        if (!lin) {
            // no query-side kernel has run: place g on the fine grid here
            e = dispatch_type_width(d.io_dtype, h->dpad, [&](auto t, auto) {
                using T = decltype(t);
                const int pieces = h->nq * (d.d / IO<T>::VEC);
                hipLaunchKernelGGL(scatter_rows_kernel<T>, dim3((pieces + 255) / 256, h->units), dim3(256),
                                   0, s, static_cast<const T*>(grad_out), static_cast<T*>(h->g_up), h->nq,
                                   d.d, d.heads, h->out_st, h->in_st, h->qgrid_w, d.grid_w);
                return hipGetLastError();
            });
            HIP_TRY(e);
        }
    }
    e = do_apply(h, true, k, g_fine, dw ? h->wflip : nullptr, nullptr, grad_v, s);
    h->ov.on = false;
    h->apply_ready = false;
    HIP_TRY(e);
    if (dw) {
        e = typed([&](auto t, auto dc) {
            size_t unused = 0;
            return bwd_filter<decltype(t), decltype(dc)::value>(h, true, v, g_fine, &unused, s);
        });
        HIP_TRY(e);
        const int n = d.heads * d.d * (taps + 1);
        hipLaunchKernelGGL(bwd_filter_combine_kernel, dim3((n + 15) / 16), dim3(256), 0, s, h->fpart,
                           grad_w, grad_bias, d.B, d.heads, d.d, h->dpad, taps, h->filter_chunks);
        HIP_TRY(hipGetLastError());
    } else {
        if (grad_w) {
            const int n = d.heads * d.d * taps;
            hipLaunchKernelGGL(fill_zero_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, grad_w, n);
        }
        if (grad_bias) {
            const int n = d.heads * d.d;
            hipLaunchKernelGGL(fill_zero_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, grad_bias, n);
        }
        HIP_TRY(hipGetLastError());
    }
    return CASTLING_OK;
}

int castling_attn_get_state(castling_attn_t h, void* host_f32, size_t bytes, void* stream)
{
    if (!h || !host_f32 || !h->state_valid) return CASTLING_ERR_INVALID_ARG;
    const int D = h->desc.d, D1 = D + 1, P = h->dpad;  // the workspace holds width-P records
    if (bytes != sizeof(float) * static_cast<size_t>(h->units) * D1 * D1)
        return CASTLING_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // no exception may leave through the C boundary: plain allocation, checked
    const size_t raw_n = static_cast<size_t>(h->units) * h->state_size;
    std::unique_ptr<float[]> raw(new (std::nothrow) float[raw_n]);
    if (!raw) return hip_fail(hipErrorOutOfMemory);
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipMemcpy(raw.get(), h->state, raw_n * sizeof(float), hipMemcpyDeviceToHost));
    float* dst = static_cast<float*>(host_f32);
    for (int u = 0; u < h->units; ++u) {
        const float* r = raw.get() + static_cast<size_t>(u) * h->state_size;
        float* m = dst + static_cast<size_t>(u) * D1 * D1;
        for (int i = 0; i < D; ++i) {
            for (int j = 0; j < D; ++j) m[i * D1 + j] = r[i * P + j];
            m[i * D1 + D] = r[P * P + i];
        }
        for (int j = 0; j < D; ++j) m[D * D1 + j] = r[P * P + P + j];
        m[D * D1 + D] = static_cast<float>(h->desc.N);
    }
    return CASTLING_OK;
}

}  // extern "C"
