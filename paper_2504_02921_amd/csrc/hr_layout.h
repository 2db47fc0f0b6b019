// In-page arrangement of the document-KV pool (private to the library), shared by the kernel that
// writes pages and the kernels that read them.  Offsets are in elements of the pool dtype.
//
// A page holds 16 tokens of one (layer, kv head): a K block followed by a V block, 16 * d elements
// each, so one page is a single contiguous burst (4 KiB at d = 64, 8 KiB at d = 128 for 16-bit KV).
//   K block: token-major rows of d channels; when d is a multiple of 64 the 8-channel chunk index is
//            XORed with (t & 7), which is the LDS bank swizzle the MFMA fragment reads want, baked
//            into HBM so that a page is copied to LDS verbatim.
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

HR_HD int k_swizzle_mask(int d) { return (d % 64 == 0) ? 7 : 0; }

HR_HD int k_elem(int t, int c, int d) { return t * d + ((((c >> 3) ^ (t & k_swizzle_mask(d))) << 3) | (c & 7)); }

HR_HD int v_elem(int t, int c, int d) { return ((t >> 2) & 1) * (d * 8) + c * 8 + ((t & 3) | ((t & 8) >> 1)); }

}  // namespace hr
