// Pieces shared by the kernels that form the lookups of Alg. 2 as one-hot int8 products on the
// matrix units (scan_u8_mfma_kernel for batches of an exhaustive scan, ivfs_scan_kernel for inverted
// lists shared by several queries): register types, the zeroing of an accumulator, and the 16-entry
// nibble table from which the compressed operand of v_smfmac_i32_32x32x64_i8 is read.
#pragma once

#include "qadc_common.h"

namespace qadc {

typedef int v2i_t __attribute__((ext_vector_type(2)));
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef int v16i_t __attribute__((ext_vector_type(16)));
typedef long v8l_t __attribute__((ext_vector_type(8)));

// Sixteen accumulator registers set to zero with eight 64-bit moves written straight into the
// registers the first product accumulates in (the sparse instruction has no zero addend; left to
// itself the compiler clears them with 23 moves per step, and every vector instruction costs the
// matrix pipe its issue slot).
__device__ __forceinline__ v16i_t mfma_zero_acc()
{
    v8l_t z;
#pragma unroll
    for (int k = 0; k < 8; ++k) asm volatile("v_mov_b64 %0, 0" : "=v"(z[k]));
    return __builtin_bit_cast(v16i_t, z);
}

// Entry c of the nibble tables, written by lane c < 16: the 8 value bytes of a nibble c (byte
// 2 (c / 4) is 1: the first value of pair c / 4) and its 16 position bits (position c mod 4 for that
// value; the two positions of a pair are kept different: (0, 3) for the empty pairs).  Two tables, so
// that the two reads of a nibble stay an 8-byte and a 4-byte read that land in the operand's
// registers; entries 8 bytes apart in both, so that the 16 entries of a table lie in 32 different LDS
// banks (16 bytes apart, entries c and c + 8 shared their banks).
__device__ __forceinline__ void onehot_nibble_entry(int c, v2i_t *nibval, v2i_t *nibpos)
{
    const int pr = c >> 2, pos = c & 3;
    const int bits = (0xcccc & ~(15 << (4 * pr))) | ((pos | ((pos == 3 ? 2 : 3) << 2)) << (4 * pr));
    nibval[c] = v2i_t{pr < 2 ? 1 << (16 * pr) : 0, pr >= 2 ? 1 << (16 * (pr - 2)) : 0};
    nibpos[c] = v2i_t{bits, 0};
}

// Every byte of the result: 8 * (this lane's nibble of the code byte), the offset of the nibble's
// entries in either table.  Lanes 0..31 (half 0) take the low nibbles, lanes 32..63 the high ones: a
// rotation brings either to bits 3..6 of its byte (what it drags in from the neighbouring byte falls
// outside the mask).
__device__ __forceinline__ unsigned onehot_nibble_offsets(unsigned w, int half)
{
    return __builtin_amdgcn_alignbit(w, w, half ? 1u : 29u) & 0x78787878u;
}

}  // namespace qadc
