// Operand images of the split-precision contraction passes (gfx950): geometry and the stores that build them.
//
// A matrix whose rows a pass streams (the chunk's negatives, the chunk's edge-side operands) is kept as "images":
// per chunk-side and tile of 32 rows a plane of the rows' bf16 hi parts and a plane of their lo parts
// (v = hi + lo, hi = bf16(v), lo = bf16(v - hi)), each [32][PA bytes], a row = 32 NS bf16 values: the dk columns and
// zeros up to the next multiple of 32.  An image is one contiguous block of IMG bytes (a multiple of 1 KB).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Row pitch in bytes of a plane whose rows hold `rowb` bytes: the pitch in 4-byte banks, mod 64, must be one of
// 12, 28, 36, 52 -- then the 16 rows of a 16-byte fragment read fall into 16 different groups of 4 LDS banks, and
// the 4 rows of a transpose read into 4 different groups of 8 banks.
constexpr int sp_pitch(int rowb) {
  for (int pad = 16; pad <= 256; pad += 16) {
    const int p = ((rowb + pad) / 4) % 64;
    if (p == 12 || p == 28 || p == 36 || p == 52) return rowb + pad;
  }
  return rowb + 16;
}
constexpr int SP_TY = 32;                                  // rows per image
constexpr int sp_plane(int ns) { return SP_TY * sp_pitch(64 * ns); }
constexpr int sp_image(int ns) { return (2 * sp_plane(ns) + 1023) / 1024 * 1024; }
// Contraction steps of 32 columns (NS) and 16-column output blocks (NCB) of the instantiation that serves dk.
constexpr int sp_ns(int dk) { return dk <= 64 ? 2 : (dk <= 128 ? 4 : (dk <= 256 ? 8 : 13)); }
constexpr int sp_ncb(int dk) { return dk <= 64 ? 4 : (dk <= 112 ? 7 : (dk <= 128 ? 8 : (dk <= 208 ? 13 : (dk <= 256 ? 16 : 25)))); }

// Where the gather writes an image set: [chunk-sides][tiles][IMG].
struct SplitImages {
  char* base;           // NULL: no images are written
  int32_t pa, plane, img, tiles, dkp;
};
static inline SplitImages sp_images(char* base, int dk, int rows_per_chunk) {
  const int ns = sp_ns(dk);
  SplitImages g;
  g.base = base; g.pa = sp_pitch(64 * ns); g.plane = sp_plane(ns); g.img = sp_image(ns);
  g.tiles = (rows_per_chunk + SP_TY - 1) / SP_TY; g.dkp = 32 * ns;
  return g;
}

#ifdef __HIPCC__
// start of row `row` of chunk-side `cs` in the hi plane; the lo plane's row is g.plane bytes further
__device__ __forceinline__ char* sp_row(const SplitImages& g, int cs, int row) {
  return g.base + ((size_t)cs * g.tiles + row / SP_TY) * g.img + (row % SP_TY) * g.pa;
}
typedef __bf16 sp_bf2 __attribute__((ext_vector_type(2)));
typedef __bf16 sp_bf4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void sp_store1(char* hi_row, int plane, int col, float v) {
  const __bf16 h = (__bf16)v;
  *reinterpret_cast<__bf16*>(hi_row + 2 * col) = h;
  *reinterpret_cast<__bf16*>(hi_row + plane + 2 * col) = (__bf16)(v - (float)h);
}
__device__ __forceinline__ void sp_store2(char* hi_row, int plane, int col, float2 v) {
  const sp_bf2 h = {(__bf16)v.x, (__bf16)v.y};
  const sp_bf2 l = {(__bf16)(v.x - (float)h[0]), (__bf16)(v.y - (float)h[1])};
  *reinterpret_cast<sp_bf2*>(hi_row + 2 * col) = h;
  *reinterpret_cast<sp_bf2*>(hi_row + plane + 2 * col) = l;
}
__device__ __forceinline__ void sp_store4(char* hi_row, int plane, int col, float4 v) {
  const sp_bf4 h = {(__bf16)v.x, (__bf16)v.y, (__bf16)v.z, (__bf16)v.w};
  const sp_bf4 l = {(__bf16)(v.x - (float)h[0]), (__bf16)(v.y - (float)h[1]), (__bf16)(v.z - (float)h[2]), (__bf16)(v.w - (float)h[3])};
  *reinterpret_cast<sp_bf4*>(hi_row + 2 * col) = h;
  *reinterpret_cast<sp_bf4*>(hi_row + plane + 2 * col) = l;
}
#endif
