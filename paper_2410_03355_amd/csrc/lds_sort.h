// Bitonic sort of a workgroup's elements in LDS, shared by the neighbour-table builds (Algorithm 2,
// precompute part: the sorted neighbour list of a token).
#pragma once

#include <hip/hip_runtime.h>

#include "device_utils.h"

namespace lantern {

// Element e of a sorted array lives in slot lds_slot(e): bits 5 and 6 of e are folded into the low
// five bits (bit 6 into bits 0, 2, 4, bit 5 into bits 1, 3).  The sort's threads read four elements
// base + q h each; whichever power of two h is, the 32 lanes of an 8-byte access then fall into
// 32 different bank pairs, where the plain layout has them collide four at a time for small h.
// The map is linear over exclusive-or and stays inside aligned blocks of 128 slots, so the array's
// length must be a multiple of 128.
__device__ __forceinline__ int lds_slot(int e) { return e ^ ((e & 64) ? 21 : 0) ^ ((e & 32) ? 10 : 0); }

// Sorts elements 0 .. P-1 (P a power of two, P >= 4, a multiple of 128 or at most 128) ascending, in
// place, by all TNT threads of the workgroup; ends with a workgroup barrier.
//   E                 an element as held in registers
//   ld(slot) -> E, st(slot, E)   access to the element stored in slot lds_slot(e)
//   after(a, b)       a orders after b (a strict total order; written without short-circuit
//                     operators, from which the compiler makes nested branches)
//   pick(sw, a, b)    b if sw, else a
//
// Four elements per thread and round trip through the LDS: for two consecutive strides 2h and h
// of a merge, thread g takes the elements base, base + h, base + 2h, base + 3h (base: g with two
// zero bits put in at the strides' places) and does both steps on them in registers; a merge with
// an odd number of steps ends with a step of stride 1 on four consecutive elements.  A
// wavefront's 64 threads cover 256 consecutive elements as long as 4h <= 256, and the same 256
// from step to step, so such a step needs the wavefront's own LDS order, not a workgroup
// barrier, unless the step before it was a wider one.
// Up to 256 elements the network runs a pair per thread and step instead (element l = 2t - t mod
// stride against l + stride): four per thread would leave all but half a wavefront idle, and the
// steps are then short enough for their number not to matter.  A wavefront's pairs stay inside
// its own blocks of 128 elements for strides up to 64.
template <int TNT, typename E, typename LD, typename ST, typename AFTER, typename PICK>
__device__ __forceinline__ void bitonic_sort_lds(int P, int tid, LD ld, ST st, AFTER after, PICK pick) {
    auto exchange = [&](E& a, E& b, bool up) {
        const bool sw = after(a, b) == up;
        const E x = pick(sw, a, b), y = pick(sw, b, a);
        a = x;
        b = y;
    };
    bool wide_before = true;   // no step yet: the elements were written by other wavefronts
    auto order_lds = [&](bool wide) {
        if (wide || wide_before) {
            __syncthreads();
        } else {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        wide_before = wide;
    };
    if (P <= 256) {
        for (int size = 2; size <= P; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                order_lds(stride > WAVE);
                const int t = tid;
                if (t < (P >> 1)) {
                    const int l = 2 * t - (t & (stride - 1));
                    const bool up = (l & size) == 0;
                    const int pl = lds_slot(l), pr = pl ^ lds_slot(stride);
                    const E a = ld(pl), b = ld(pr);
                    if (after(a, b) == up) {
                        st(pl, b);
                        st(pr, a);
                    }
                }
            }
        }
    }
    for (int size = 2, m = 1; P > 256 && size <= P; size <<= 1, ++m) {
        int J = m - 1;   // the widest stride still to do in this merge is 2^J
        for (; J >= 1; J -= 2) {
            order_lds(J + 1 > 8);
            const int h = 1 << (J - 1);
            for (int g = tid; g < (P >> 2); g += TNT) {
                const int base = ((g >> (J - 1)) << (J + 1)) | (g & (h - 1));
                const bool up = (base & size) == 0;
                // base has zero bits where h and 2h have theirs, and lds_slot is linear
                const int p0 = lds_slot(base), p1 = p0 ^ lds_slot(h), p2 = p0 ^ lds_slot(2 * h), p3 = p0 ^ lds_slot(3 * h);
                E e0 = ld(p0), e1 = ld(p1), e2 = ld(p2), e3 = ld(p3);
                exchange(e0, e2, up);
                exchange(e1, e3, up);
                exchange(e0, e1, up);
                exchange(e2, e3, up);
                st(p0, e0); st(p1, e1); st(p2, e2); st(p3, e3);
            }
        }
        if (J == 0) {
            order_lds(false);
            for (int g = tid; g < (P >> 2); g += TNT) {
                const int base = 4 * g;
                const int p0 = lds_slot(base), p1 = p0 ^ 1, p2 = p0 ^ 2, p3 = p0 ^ 3;
                E e0 = ld(p0), e1 = ld(p1), e2 = ld(p2), e3 = ld(p3);
                exchange(e0, e1, (base & size) == 0);
                exchange(e2, e3, ((base + 2) & size) == 0);
                st(p0, e0); st(p1, e1); st(p2, e2); st(p3, e3);
            }
        }
    }
    __syncthreads();
}

}  // namespace lantern
