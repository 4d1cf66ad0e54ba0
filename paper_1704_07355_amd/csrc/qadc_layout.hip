// Conversion between the two list layouts of the paper's Fig. 2 (Section 3.2) on gfx950.
//
// Standard layout: code i = m/2 consecutive bytes.  Transposed layout: each block of 16 codes is
// stored as m/2 rows of 16 bytes, row j holding byte j of the 16 codes; the last block is filled
// with zero bytes.  The paper transposes lists offline so that one 128-bit register holds one
// component of 16 codes; the scan kernels of this library read the standard layout (a lane's
// 16-byte load is already the unit of coalescing), so a database kept in the transposed layout
// is converted once with qadc_unpack_codes, and qadc_pack_codes writes one for programs that
// scan block by block.
//
// Both directions move 16-byte pieces through LDS: a workgroup of 256 threads handles 256 pieces
// (256 / (m/2) blocks), reads them with one 16-byte load per thread, and every thread gathers the
// 16 bytes of one output piece.  Memory-bound: one read and one write of the list.

#include "qadc_common.h"

namespace qadc {

constexpr int LAYOUT_NT = 256;

// TO_T: standard -> transposed, else transposed -> standard.  B = m/2 divides 256.
// Piece p of a block (16 B): bytes [16p, 16p+16) of the block's 16*B bytes in either layout.
template <bool TO_T>
__global__ __launch_bounds__(LAYOUT_NT) void relayout_kernel(const uint8_t *__restrict__ src, int64_t n,
                                                              int B, uint8_t *__restrict__ dst)
{
    __shared__ __attribute__((aligned(16))) uint8_t tile[LAYOUT_NT * 16];
    const int tid = threadIdx.x;
    const int64_t piece = (int64_t)blockIdx.x * LAYOUT_NT + tid;   // global 16-byte piece
    const int64_t std_bytes = n * B;                                // bytes of the standard list
    const int64_t nblk = (n + 15) / 16;
    const int64_t pieces = nblk * B;
    // load: a piece of the source layout, zero beyond the source's end
    uint4 v = make_uint4(0, 0, 0, 0);
    if (piece < pieces) {
        const int64_t off = piece * 16;
        if (!TO_T || off + 16 <= std_bytes) {
            v = *reinterpret_cast<const uint4 *>(src + off);
        } else if (off < std_bytes) {  // the standard list ends inside this piece
            uint8_t b[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) b[e] = (off + e < std_bytes) ? src[off + e] : (uint8_t)0;
            v = *reinterpret_cast<const uint4 *>(b);
        }
    }
    reinterpret_cast<uint4 *>(tile)[tid] = v;
    __syncthreads();
    if (piece >= pieces) return;
    // gather: output piece p of local block lb
    const int lb = tid / B, p = tid - lb * B;
    const uint8_t *blk = tile + lb * 16 * B;
    uint8_t o[16];
    if (TO_T) {
        // row p of the block: byte p of codes 0..15, code c at blk[c*B + p]
#pragma unroll
        for (int c = 0; c < 16; ++c) o[c] = blk[c * B + p];
    } else {
        // bytes [16p, 16p+16) of the standard block: byte q = code q / B, row q % B -> blk[row*16 + code]
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int q = 16 * p + e;
            const int c = q / B, r = q - c * B;
            o[e] = blk[r * 16 + c];
        }
    }
    const int64_t off = piece * 16;
    if (TO_T || off + 16 <= std_bytes) {
        *reinterpret_cast<uint4 *>(dst + off) = *reinterpret_cast<const uint4 *>(o);
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (off + e < std_bytes) dst[off + e] = o[e];
    }
}

static bool layout_m_ok(int m) { return m == 8 || m == 16 || m == 32 || m == 64; }

size_t packed_bytes(int64_t n, int m, int layout)
{
    if (n < 0 || !layout_m_ok(m)) return 0;
    if (layout == QADC_LAYOUT_STANDARD) return (size_t)n * (size_t)(m / 2);
    if (layout == QADC_LAYOUT_TRANSPOSED) return (size_t)((n + 15) / 16) * 16 * (size_t)(m / 2);
    return 0;
}

int relayout(bool pack, const uint8_t *src, int64_t n, int m, int layout, uint8_t *dst, hipStream_t st)
{
    const char *name = pack ? "qadc_pack_codes" : "qadc_unpack_codes";
    if (n < 0 || !layout_m_ok(m)) return fail(QADC_EINVAL, "%s: unsupported n=%lld m=%d", name, (long long)n, m);
    if (layout != QADC_LAYOUT_STANDARD && layout != QADC_LAYOUT_TRANSPOSED)
        return fail(QADC_EINVAL, "%s: unknown layout %d", name, layout);
    if (n == 0) return QADC_OK;
    if (!src || !dst) return fail(QADC_EINVAL, "%s: null pointer", name);
    if (src == dst) return fail(QADC_EINVAL, "%s: source and destination must not overlap", name);
    if (layout == QADC_LAYOUT_STANDARD) {
        QADC_HIP_TRY(hipMemcpyAsync(dst, src, (size_t)n * (m / 2), hipMemcpyDeviceToDevice, st));
        return QADC_OK;
    }
    if (((uintptr_t)src | (uintptr_t)dst) & 15)
        return fail(QADC_EINVAL, "%s: pointers must be 16-byte aligned", name);
    const int B = m / 2;
    const int64_t pieces = (n + 15) / 16 * B;
    const int64_t grid = ceil_div(pieces, LAYOUT_NT);
    if (grid > 0x7fffffffll) return fail(QADC_EINVAL, "%s: n too large for one call", name);
    if (pack)
        hipLaunchKernelGGL(relayout_kernel<true>, dim3((unsigned)grid), dim3(LAYOUT_NT), 0, st, src, n, B, dst);
    else
        hipLaunchKernelGGL(relayout_kernel<false>, dim3((unsigned)grid), dim3(LAYOUT_NT), 0, st, src, n, B, dst);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
