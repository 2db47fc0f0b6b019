// In-page arrangement of the document-KV pool (private to the library), shared by the kernel that
// writes pages and the kernels that read them.  Offsets are in elements of the pool dtype.
//
// A page holds 16 tokens of one (layer, kv head): a K block followed by a V block, 16 * d elements
// each, so one page is a single contiguous burst (4 KiB at d = 64, 8 KiB at d = 128 for 16-bit KV).
//   K block: token-major rows of d channels with the 8-channel chunk index XOR-swizzled by the token
//            index.  The swizzle is the LDS bank pattern the MFMA fragment reads want (LDS has 64 banks
//            of 4 bytes = 256 bytes per cycle, and a 16-byte read serves 16 lanes per cycle, so the 16
//            rows read together must land on 16 different 16-byte positions of that 256-byte window:
//            128-byte rows are swizzled by the row pair (t >> 1) & 7, 256-byte rows by t & 15).  It is
//            baked into HBM so that a page is copied to LDS verbatim.
//   V block: transposed and split by key parity group: [t bit 2][channel][8 keys], where the 8 keys
//            of a group are t = {0,1,2,3,8,9,10,11} (+4 for the second group).  A wavefront lane that
//            feeds v_mfma_f32_32x32x16 with V^T reads its 8 keys as one 16-byte word.
#pragma once

#if defined(__HIPCC__)
#define HR_HD __host__ __device__ __forceinline__
#else
#define HR_HD inline
#endif

namespace hr {

// esz: bytes per element of the pool dtype
HR_HD int k_swizzle(int t, int d, int esz) {
    if (esz > 2) return 0;                       // fp32 pools are only read by the generic kernels
    const int row_bytes = d * esz;
    return row_bytes == 128 ? ((t >> 1) & 7) : row_bytes == 256 ? (t & 15) : 0;
}

HR_HD int k_elem(int t, int c, int d, int esz) { return t * d + ((((c >> 3) ^ k_swizzle(t, d, esz)) << 3) | (c & 7)); }

HR_HD int v_elem(int t, int c, int d) { return ((t >> 2) & 1) * (d * 8) + c * 8 + ((t & 3) | ((t & 8) >> 1)); }

}  // namespace hr
