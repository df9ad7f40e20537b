// Instantiates the row-per-lane greedy kernel for every supported dimension of one input type.
#pragma once

#include "greedy_rpl.h"

namespace e4q {

template <typename Tin>
inline hipError_t dispatch_greedy_rpl(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    switch (dim) {
#define E4Q_CASE(D) \
    case D:         \
        return launch_greedy_rpl<D, Tin>(a, stream);
        E4Q_CASE(8)
        E4Q_CASE(16)
        E4Q_CASE(24)
        E4Q_CASE(32)
        E4Q_CASE(40)
        E4Q_CASE(48)
        E4Q_CASE(56)
        E4Q_CASE(64)
        E4Q_CASE(72)
        E4Q_CASE(80)
        E4Q_CASE(88)
        E4Q_CASE(96)
        E4Q_CASE(104)
        E4Q_CASE(112)
        E4Q_CASE(120)
        E4Q_CASE(128)
#undef E4Q_CASE
        default:
            return hipErrorInvalidValue;
    }
}

template <typename Tin>
inline hipError_t dispatch_greedy_rpl_group(const GreedyGroup& g, int32_t dim, hipStream_t stream)
{
    switch (dim) {
#define E4Q_CASE(D) \
    case D:         \
        return launch_greedy_rpl_group<D, Tin>(g, stream);
        E4Q_CASE(8)
        E4Q_CASE(16)
        E4Q_CASE(24)
        E4Q_CASE(32)
        E4Q_CASE(40)
        E4Q_CASE(48)
        E4Q_CASE(56)
        E4Q_CASE(64)
        E4Q_CASE(72)
        E4Q_CASE(80)
        E4Q_CASE(88)
        E4Q_CASE(96)
        E4Q_CASE(104)
        E4Q_CASE(112)
        E4Q_CASE(120)
        E4Q_CASE(128)
#undef E4Q_CASE
        default:
            return hipErrorInvalidValue;
    }
}

// Multiples of 8 from 136 to 224: the row still fits the registers of one lane with two waves per SIMD.
template <typename Tin>
inline hipError_t dispatch_greedy_rpl_wide(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    switch (dim) {
#define E4Q_CASE(D) \
    case D:         \
        return launch_greedy_rpl<D, Tin>(a, stream);
        E4Q_CASE(136)
        E4Q_CASE(144)
        E4Q_CASE(152)
        E4Q_CASE(160)
        E4Q_CASE(168)
        E4Q_CASE(176)
        E4Q_CASE(184)
        E4Q_CASE(192)
        E4Q_CASE(200)
        E4Q_CASE(208)
        E4Q_CASE(216)
        E4Q_CASE(224)
#undef E4Q_CASE
        default:
            return hipErrorInvalidValue;
    }
}

// Dimensions between 128 and 224 that are not multiples of 8: the kernel for the next multiple of 8.
template <typename Tin>
inline hipError_t dispatch_greedy_rpl_wide_tail(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    switch ((dim + 7) / 8 * 8) {
#define E4Q_CASE(D) \
    case D:         \
        return launch_greedy_rpl_tail<D, Tin>(a, dim, stream);
        E4Q_CASE(136)
        E4Q_CASE(144)
        E4Q_CASE(152)
        E4Q_CASE(160)
        E4Q_CASE(168)
        E4Q_CASE(176)
        E4Q_CASE(184)
        E4Q_CASE(192)
        E4Q_CASE(200)
        E4Q_CASE(208)
        E4Q_CASE(216)
        E4Q_CASE(224)
#undef E4Q_CASE
        default:
            return hipErrorInvalidValue;
    }
}

// Dimensions below 128 that are not multiples of 8: the kernel for the next multiple of 8.
template <typename Tin>
inline hipError_t dispatch_greedy_rpl_tail(const GreedyArgs& a, int32_t dim, hipStream_t stream)
{
    switch ((dim + 7) / 8 * 8) {
#define E4Q_CASE(D) \
    case D:         \
        return launch_greedy_rpl_tail<D, Tin>(a, dim, stream);
        E4Q_CASE(8)
        E4Q_CASE(16)
        E4Q_CASE(24)
        E4Q_CASE(32)
        E4Q_CASE(40)
        E4Q_CASE(48)
        E4Q_CASE(56)
        E4Q_CASE(64)
        E4Q_CASE(72)
        E4Q_CASE(80)
        E4Q_CASE(88)
        E4Q_CASE(96)
        E4Q_CASE(104)
        E4Q_CASE(112)
        E4Q_CASE(120)
        E4Q_CASE(128)
#undef E4Q_CASE
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace e4q
