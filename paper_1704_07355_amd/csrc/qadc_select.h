// Workgroup-level exact selection: the r-th smallest key of a list by radix
// select (one 256-bin histogram pass per key byte, most significant first).
// Keys are unsigned integers whose order is the wanted order; for the scans a
// key is (distance << index_bits) | index, so the r-th smallest key is the r-th
// neighbour under the total order (distance, index) and keys are unique.
#pragma once

#include "qadc_common.h"

namespace qadc {

constexpr int SELECT_SMALL = 64;  // keys left in the race that one wavefront ranks directly

struct SelectScratch {
    unsigned hist[256];
    unsigned bin;
    unsigned need;
    unsigned nsmall;
    unsigned long long small[SELECT_SMALL];
    unsigned long long result;
};

// Scan of a 256-bin histogram by the first wave: finds the bin holding the
// `need`-th smallest element (1-based) and the rank of that element inside the bin
// (the last element when fewer than `need` were counted).
__device__ __forceinline__ void select_bin(SelectScratch *sc, unsigned need)
{
    if (threadIdx.x < WAVE) {
        const int l = lane_id();
        unsigned h0 = sc->hist[4 * l + 0], h1 = sc->hist[4 * l + 1];
        unsigned h2 = sc->hist[4 * l + 2], h3 = sc->hist[4 * l + 3];
        unsigned tot = h0 + h1 + h2 + h3;
        unsigned inc = tot;
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            unsigned up = __shfl_up(inc, d);
            if (l >= d) inc += up;
        }
        // a request beyond the histogram's total is answered with its last element, an empty
        // histogram with bin 0 and rank 0: the result is defined for every input
        const unsigned total = __shfl(inc, WAVE - 1);
        if (need > total) need = total;
        if (need == 0 && l == 0) { sc->bin = 0; sc->need = 0; }
        unsigned excl = inc - tot;
        unsigned h[4] = {h0, h1, h2, h3};
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (excl < need && need <= excl + h[b]) {
                sc->bin = 4 * l + b;
                sc->need = need - excl;
            }
            excl += h[b];
        }
    }
}

// The `need`-th smallest (1-based) of the keys enumerated by `each`, a callable that the
// whole workgroup calls as each(f) and that invokes f(key) once per key, spread over the
// threads in any way.  At least `need` keys must exist.  Every thread of the workgroup must
// call this with the same arguments; every thread gets the result.  NBYTES = number of
// low key bytes that can be non-zero.
template <typename K, int NBYTES, typename Each>
__device__ K block_radix_select_each(Each each, unsigned need, SelectScratch *sc)
{
    K prefix = 0, mask = 0;
    for (int shift = (NBYTES - 1) * 8; shift >= 0; shift -= 8) {
        for (unsigned i = threadIdx.x; i < 256; i += blockDim.x) sc->hist[i] = 0;
        __syncthreads();
        each([&](K k) {
            if ((k & mask) == prefix) atomicAdd(&sc->hist[(unsigned)(k >> shift) & 255u], 1u);
        });
        __syncthreads();
        select_bin(sc, need);
        __syncthreads();
        need = sc->need;
        const unsigned left = sc->hist[sc->bin];  // keys that share the prefix found so far
        prefix |= (K)sc->bin << shift;
        mask |= (K)255 << shift;
        if (threadIdx.x == 0) sc->nsmall = 0;
        __syncthreads();
        if (shift > 0 && need >= 1u && left >= need && left <= (unsigned)SELECT_SMALL) {  // uniform
            // A handful of keys left (equal ones included): they are gathered and one wavefront finds
            // the need-th smallest among them by counting, instead of a histogram pass per byte left.
            each([&](K k) {
                if ((k & mask) == prefix) sc->small[atomicAdd(&sc->nsmall, 1u)] = (unsigned long long)k;
            });
            __syncthreads();
            if (threadIdx.x < WAVE) {
                const unsigned n = sc->nsmall;
                const unsigned l = threadIdx.x;
                const unsigned long long mine = l < n ? sc->small[l] : ~0ull;
                unsigned less = 0, leq = 0;
                for (unsigned j = 0; j < n; ++j) {
                    const unsigned long long o = sc->small[j];
                    less += o < mine ? 1u : 0u;
                    leq += o <= mine ? 1u : 0u;
                }
                if (l < n && less < need && need <= leq) sc->result = mine;  // (equal keys write the same value)
            }
            __syncthreads();
            return (K)sc->result;
        }
    }
    return prefix;
}

// Same over a flat array keys[0..cnt) in LDS or global memory (need <= cnt).
template <typename K, int NBYTES>
__device__ K block_radix_select(const K *keys, unsigned cnt, unsigned need, SelectScratch *sc)
{
    return block_radix_select_each<K, NBYTES>(
        [&](auto f) {
            for (unsigned i = threadIdx.x; i < cnt; i += blockDim.x) f(keys[i]);
        },
        need, sc);
}

}  // namespace qadc
