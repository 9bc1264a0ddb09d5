// Declarations shared by the contraction kernels' translation units (gfx950): the argument block of a launch, the
// matrix-instruction wrappers and the buffer-load helpers.
#pragma once
#include "mar_common.h"

typedef float v4f __attribute__((ext_vector_type(4)));


struct FlashArgs {
  const float* X;      // stationary matrix, rows of dk floats
  const float* Y;      // streamed matrix
  const float* xx;     // squared row norms (TransE)
  const float* yy;
  float* ml;           // [sy1][2][B][2]: per part, the softmax reference and the sum of exp(score - reference);
                       // written by pass 1, combined into the log-sum-exp by pass 2
  const float* pos;    // [B] positive scores (pass 3)
  float* out;          // pass 1: unnormalised gQ rows [sy][2][B][dk]; pass 2: gradient rows G
  int32_t* rank_dst; int32_t* rank_src;   // pass 3
  int32_t n, B, C, N, S, cn, nchunks, dk, nstripes;
  int32_t sy;          // workgroups sharing one stripe, each streaming `tps` tiles
  int32_t tps;
  int32_t sy_ml;       // parts pass 1 was split into
  // pass 1 of a full batch: workgroup slots (per XCD) from whole_slots on take the stripes of chunk-sides
  // rem_cs0.. in rem_k parts of rem_tps tiles each; parts 1.. write to mlx / outx [part - 1][rem_rows]
  int32_t whole_slots, rem_cs0, rem_k, rem_tps;
  int64_t rem_rows;
  float* mlx; float* outx;
  int32_t roles;       // edge-side occurrences per edge (3, or 2 for Dot)
  float* T;            // [2*nchunks][trows][tpitch] softmax weight exp(score - reference) of every (edge, negative)
                       // pair (TransE: divided by the distance): written by pass 1, read by the negatives' gradient
                       // pass, which then needs no score product and no exponential
  float* R;            // [2*nchunks][tpitch/16][trows] the reference pass 1 used for a 16-negative block of an edge
  int32_t tpitch;      // N rounded up to 128 (whole tiles of pass 1 and whole stripes of pass 2)
  int32_t trows;       // chunk size rounded up to 64
  // split-precision passes: bf16 hi/lo images of the streamed matrix, [2*nchunks][yimg_tiles][image bytes]
  const char* yimg; int32_t yimg_tiles;
  const char* ximg; int32_t ximg_tiles;   // the same of the stationary matrix
};

__device__ __forceinline__ v4f mfma16(float a, float b, v4f c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
// Sixteen 4x4 outer products, one per group of 4 consecutive lanes: lane 4q + j, register i gets
// a(lane 4q + i) * b(lane 4q + j) added.  Used for the last 4 output columns of the second product when the
// width leaves 4 columns over the 16-wide blocks: with a = Y[y][16 NC + (lane & 3)] and b = W[y][x] of the
// lane's own (y, x), register i accumulates column 16 NC + i of O^T[.][x] over the lane's own streamed rows.
__device__ __forceinline__ v4f mfma4(float a, float b, v4f c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}

// Streamed operands are fetched with buffer loads: a descriptor (base, size in bytes) in scalar registers, a
// per-lane byte offset that never changes and a scalar byte offset that moves from tile to tile, so the tile
// loops hold no per-lane address arithmetic.  A load whose offset lies at or beyond the size returns 0 without
// touching memory (the descriptor's range check), which stands in for every "row beyond the chunk" test.
// Word 3 of the descriptor: 32-bit data format, linear addressing.
typedef __amdgpu_buffer_rsrc_t BufRsrc;
__device__ __forceinline__ BufRsrc buf_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ v4f buf_load4(BufRsrc r, int voff, int soff) {
  return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
}
__device__ __forceinline__ float2 buf_load2(BufRsrc r, int voff, int soff) {
  return __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
}
__device__ __forceinline__ float buf_load1(BufRsrc r, int voff, int soff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
#define MAR_BUF_NOWHERE 0x40000000                        // a per-lane offset beyond every descriptor's size: loads 0
// The same load with LDS as its destination: lane i's 16 bytes land at LDS byte address lds_addr + 16 i, without
// passing through registers (zeros beyond the descriptor's size).  Written as an instruction so that the compiler
// does not make every later LDS read wait for it; its completion is observed through a register load issued
// behind it (memory operations of a wave complete in order).  The descriptor is given as its four words.
typedef int v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4i buf_words(const void* base, uint32_t bytes) {
  const unsigned long long b = (unsigned long long)base;
  return (v4i){(int)(unsigned)b, (int)((unsigned)(b >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
// `token` ties later code to the instruction: a value that passes through it unchanged.
__device__ __forceinline__ void buf_load4_to_lds(v4i words, unsigned lds_addr, int voff, int soff, int& token) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, %4 offen lds"
               : "+v"(token) : "s"(lds_addr), "v"(voff), "s"(words), "s"(soff));
}
__device__ __forceinline__ unsigned lds_address(const float* p) {
  return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const float*)p;
}

// Waves per SIMD a kernel is built for: the register allocator may use the whole share of the register file
// that this occupancy leaves to a wave, and does not trade spills for a higher occupancy.
#define MAR_WAVES_PER_SIMD(n) __attribute__((amdgpu_waves_per_eu(n, n)))

// Launch of a split-precision pass (mar_split.hip); `a` as filled by mar_launch_flash.
hipError_t mar_split_launch(const FlashArgs& a, int pass, dim3 grid, hipStream_t st);
