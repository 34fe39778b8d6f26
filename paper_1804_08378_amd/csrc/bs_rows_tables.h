// Signatures (pooling shapes and element-wise lists) the sliding-window kernels are compiled
// into the library for; any other signature is built at plan time.  Host only; shared by the
// kernels that load their edge columns and the ones that exchange them between lanes.
#pragma once
#include <type_traits>

#include "bs_rows_device.h"

namespace bs {

template <int V>
using IC = std::integral_constant<int, V>;

// one-level kernels: F(pool, pre code, post code) returns true to stop
template <class F>
static bool rows_for_each_signature(F &&f)
{
    return f(RMax3s2p1{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{}) ||
           f(RMax3s2p1{}, IC<RW_NONE>{}, IC<RW_NONE>{}) ||
           f(RMax3s2p0{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{}) ||
           f(RMax3s2p0{}, IC<RW_NONE>{}, IC<RW_NONE>{}) ||
           f(RMax3s2p0{}, IC<RW_RELU>{}, IC<RW_NONE>{}) ||
           f(RMax3s2p1{}, IC<RW_RELU>{}, IC<RW_NONE>{}) ||
           f(RMax3s1p1{}, IC<RW_NONE>{}, IC<RW_BN_RELU>{}) ||
           f(RMax3s1p1{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{}) ||
           f(RMax3s1p1{}, IC<RW_NONE>{}, IC<RW_NONE>{}) ||
           f(RAvg3s1p1{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{}) ||
           f(RAvg3s1p1{}, IC<RW_NONE>{}, IC<RW_NONE>{});
}

// two-level kernels: F(pool 1, pool 2, code 0, code 1, code 2) returns true to stop
template <class F>
static bool rows2_for_each_signature(F &&f)
{
    return f(RAvg3s1p1{}, RMax3s2p1{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{}, IC<RW_BN_RELU>{}) ||
           f(RMax3s1p1{}, RMax3s1p1{}, IC<RW_NONE>{}, IC<RW_BN_RELU>{}, IC<RW_BN_RELU>{}) ||
           f(RMax3s1p1{}, RAvg3s1p1{}, IC<RW_NONE>{}, IC<RW_BN_RELU>{}, IC<RW_NONE>{});
}

}  // namespace bs
