// Scaffolding shared by the tiled matrix-product kernels (gemm_fast.hip, gemm_mid.hip, gemm_f8.hip,
// gemm_ws.hip): which tile a workgroup owns, the buffer descriptors of the two code tensors, the image
// position of an output pixel, and the counter that walks a convolution's K steps through the filter taps.
#ifndef DYBIT_TILE_COMMON_H
#define DYBIT_TILE_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dybit_codec.h"
#include "gemm_args.h"

namespace dybit {
namespace fast {

// Position of this workgroup in the tile order.  Workgroup ids go round-robin over the 8 XCDs, so XCD x
// (id mod 8) is given the contiguous range [x per_xcd, (x + 1) per_xcd) of the order: the tiles it has in
// flight are neighbours and share their operand strips in its own L2.  The grid is a multiple of 8.
__device__ __forceinline__ int xcd_contiguous_index()
{
    const int per_xcd = (int)gridDim.x >> 3;
    return ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
}

// Tile order that walks column panels of up to 8 tiles row by row (the 32 tiles of an XCD form a compact
// 4 x 8 patch).  Returns false when index l has no tile (uniform per workgroup).
__device__ __forceinline__ bool panel_order_tile(int l, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    if (l >= tiles_m * tiles_n) return false;
    const int panel = l / (tiles_m * 8), r = l - panel * tiles_m * 8;
    const int width = min(8, tiles_n - panel * 8);             // the last panel may be narrower
    tile_m = r / width;
    tile_n = panel * 8 + (r - tile_m * width);
    return true;
}

// Row-major tile order (all column tiles of a row strip together).
__device__ __forceinline__ bool row_order_tile(int l, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    if (l >= tiles_m * tiles_n) return false;
    tile_m = l / tiles_n;
    tile_n = l - tile_m * tiles_n;
    return true;
}

// Raw buffer descriptor over a tensor of packed codes (byte offsets, range-checked by the hardware: a load
// at or past `bytes`, in particular at kOob, returns 0 = code 0).  Tensors beyond 2 GiB are clamped; the
// dispatcher does not send them here.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t code_descriptor(const uint8_t *p, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p), 0, (int)(bytes > 0x7fffffff ? 0x7fffffff : bytes), 0x00020000);
}

// Output pixel m of a convolution: the image row and column of its filter tap (0, 0) (negative inside the
// padding) and the pixel index of that tap in the NHWC image, (b H + hi0) Wd + wi0 (may be negative).
struct PixelOrigin {
    int hi0, wi0;
    int64_t first_pixel;
};
__device__ __forceinline__ PixelOrigin pixel_origin(const GemmArgs &g, int64_t m)
{
    const int b = (int)(m / ((int64_t)g.Ho * g.Wo));
    const int rem = (int)(m - (int64_t)b * g.Ho * g.Wo);
    const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
    PixelOrigin o;
    o.hi0 = ho * g.stride - g.pad;
    o.wi0 = wo * g.stride - g.pad;
    o.first_pixel = ((int64_t)b * g.H + o.hi0) * g.Wd + o.wi0;
    return o;
}

// K steps of a convolution are loaded in order, so the filter row, filter column and first channel of the
// next step are counted up instead of being divided out of k every time (k = (fr kw + fs) Cin + c0).
struct TapCounter {
    int fr = 0, fs = 0, c0 = 0;
    __device__ __forceinline__ void advance(int codes, const GemmArgs &g)
    {
        c0 += codes;
        while (c0 >= g.Cin) {
            c0 -= g.Cin;
            if (++fs == g.kw) { fs = 0; ++fr; }
        }
    }
    // byte offset of the tap's channel c0 from the pixel's tap (0, 0)
    __device__ __forceinline__ int byte_offset(const GemmArgs &g, int pix_bytes, int bits) const
    {
        return (fr * g.Wd + fs) * pix_bytes + c0 * bits / 8;
    }
    __device__ __forceinline__ bool inside(const GemmArgs &g, int hi0, int wi0) const
    {
        return (unsigned)(hi0 + fr) < (unsigned)g.H && (unsigned)(wi0 + fs) < (unsigned)g.Wd;
    }
};

}  // namespace fast
}  // namespace dybit
#endif
