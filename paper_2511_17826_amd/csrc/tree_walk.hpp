// The in-kernel part of the tree (App. C operator T by the carry-over scheme of App. D.1, Alg. 1) over a workgroup
// tile's accumulators: shared by the tiled GEMM kernels of every operand format.
#pragma once

#include "tbik_device.hpp"

namespace tbik {

template <int MT, int NT>              // 32x32 MFMA tiles per wavefront
struct Acc {
    f32x16 t[MT][NT];
};

// Stash of finished subtrees (App. D.1: accumulator buffer S[level]) for tree levels 1 and up; every slot
// is addressed statically, so the slots are registers.  Level 0 needs no slot: two consecutive superleaves
// are accumulated in two different register sets and added.
template <int SLOTS, int MT, int NT>
struct TileStash {
    Acc<MT, NT> s[SLOTS > 0 ? SLOTS : 1];
};

template <int MT, int NT>
__device__ __forceinline__ void add_left_sibling(Acc<MT, NT> &acc, const Acc<MT, NT> &left) {
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc.t[a][b][r] = left.t[a][b][r] + acc.t[a][b][r];
}

// Evaluates T over 2^L consecutive superleaves into acc (App. C), leaves in ascending k.  The walk is a
// nest of two-trip loops: the first trip of the loop at level l parks its subtree sum in slot l, the
// second trip adds the slot to its own sum (left sibling + right sibling).
template <int L>
struct SubtreeWalker {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, A &acc2, S &stash) {
#pragma nounroll
        for (int half = 0; half < 2; ++half) {
            SubtreeWalker<L - 1>::run(leaf, acc, acc2, stash);
            if (half == 0) stash.s[L - 2] = acc;
            else add_left_sibling(acc, stash.s[L - 2]);
        }
    }
};
template <>
struct SubtreeWalker<1> {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, A &acc2, S &) {
        leaf(acc);                       // superleaf 2i   -> first register set
        leaf(acc2);                      // superleaf 2i+1 -> second register set
        add_left_sibling(acc2, acc);     // left + right
        acc = acc2;
    }
};
template <>
struct SubtreeWalker<0> {
    template <class Leaf, class A, class S>
    __device__ __forceinline__ static void run(Leaf &leaf, A &acc, A &, S &) { leaf(acc); }
};

}  // namespace tbik
