// Instantiations and launchers of the one-launch forward (stream_fwd.hpp).
#include "stream_fwd_host.hpp"

namespace castling {

void build_stream_tasks(int units, int cr, int ca, int ncs, int nw, int lookahead, bool lin,
                        std::vector<uint32_t>& tasks, uint32_t (&queue_off)[kStreamQueues + 1])
{
    tasks.clear();
    for (int x = 0; x < kStreamQueues; ++x) {
        queue_off[x] = static_cast<uint32_t>(tasks.size());
        for (int i = x; i < nw; i += kStreamQueues) tasks.push_back(make_task(kTaskWeights, 0, i));
        std::vector<int> mine;
        for (int u = x; u < units; u += kStreamQueues) mine.push_back(u);
        const int U = static_cast<int>(mine.size());
        auto combine = [&](int u) {
            for (int i = 0; i < ncs; ++i) tasks.push_back(make_task(kTaskCombine, u, i));
        };
        if (lin)
            for (int jj = 0; jj < std::min(lookahead, U); ++jj) {
                for (int i = 0; i < cr; ++i) tasks.push_back(make_task(kTaskReduce, mine[jj], i));
                combine(mine[jj]);
            }
        for (int jj = 0; jj < U; ++jj) {
            const int jr = jj + lookahead;
            const bool more = lin && jr < U;
            const int n = std::max(ca, more ? cr : 0);
            // apply chunk i * ca / n and reduce chunk i * cr / n: both lists dealt evenly over n rounds
            int ia = 0, ir = 0;
            for (int i = 0; i < n; ++i) {
                if (ia < ca && static_cast<long long>(ia) * n <= static_cast<long long>(i) * ca)
                    tasks.push_back(make_task(kTaskApply, mine[jj], ia++));
                if (more && ir < cr && static_cast<long long>(ir) * n <= static_cast<long long>(i) * cr)
                    tasks.push_back(make_task(kTaskReduce, mine[jr], ir++));
            }
            for (; ia < ca; ++ia) tasks.push_back(make_task(kTaskApply, mine[jj], ia));
            for (; more && ir < cr; ++ir) tasks.push_back(make_task(kTaskReduce, mine[jr], ir));
            if (more) combine(mine[jr]);
        }
    }
    queue_off[kStreamQueues] = static_cast<uint32_t>(tasks.size());
}

namespace {

template <typename F>
hipError_t with_kernel(int ks, bool lin, bool dw, bool half, F&& f)
{
    auto with_fmt = [&](auto ks_c, auto lin_c, auto dw_c) {
        constexpr int KS = decltype(ks_c)::value;
        constexpr bool LIN = decltype(lin_c)::value, DW = decltype(dw_c)::value;
        return half ? f(&stream_forward_kernel<KS, LIN, DW, F16Fmt>)
                    : f(&stream_forward_kernel<KS, LIN, DW, Bf16Fmt>);
    };
    auto with_branches = [&](auto ks_c) {
        using T = std::true_type;
        using N = std::false_type;
        if (lin && dw) return with_fmt(ks_c, T{}, T{});
        if (lin) return with_fmt(ks_c, T{}, N{});
        return with_fmt(ks_c, N{}, T{});
    };
#ifdef CASTLING_STREAM_ONLY_KS
    return with_branches(std::integral_constant<int, CASTLING_STREAM_ONLY_KS>{});
#else
    switch (ks) {
        case 1: return with_branches(std::integral_constant<int, 1>{});
        case 3: return with_branches(std::integral_constant<int, 3>{});
        case 5: return with_branches(std::integral_constant<int, 5>{});
        case 7: return with_branches(std::integral_constant<int, 7>{});
        default: return with_branches(std::integral_constant<int, 9>{});
    }
#endif
}

}  // namespace

hipError_t stream_forward_prepare(int ks, bool lin, bool dw, bool half, int* blocks_per_cu)
{
    return with_kernel(ks, lin, dw, half, [&](auto kernel) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kStreamLdsBytes);
        if (e != hipSuccess) return e;
        return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, kernel, 256, kStreamLdsBytes);
    });
}

hipError_t stream_forward_launch(int ks, bool lin, bool dw, bool half, const StreamArgs& a, int blocks,
                                 hipStream_t s)
{
    return with_kernel(ks, lin, dw, half, [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), kStreamLdsBytes, s, a);
        return hipGetLastError();
    });
}

}  // namespace castling
