// Shared device-side definitions of the gfx950 Video Sparse Attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vsa {

constexpr int kTile = 64;  // rows of one attention block; a cube of V = 64*m tokens (Sec. 2.2: V = 4*4*4;
                           // Sec. 3.2 ablates 128 and 256) is m consecutive blocks of the tiled order

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Geometry of the padded latent grid (Sec. 2.2), passed to kernels by value.
struct Geo {
  int T, Hh, W;     // valid grid
  int Ct, Ch, Cw;   // cube
  int Nt, Nh, Nw;   // cubes per axis
  int Nc;           // cubes
  int V, m;         // tokens per cube, 64-row blocks per cube (V = 64 * m)
  int Nb;           // blocks = Nc * m
  int L;            // valid tokens
  long long Np;     // padded tokens = V * Nc
};

// bf16 bits <-> fp32.  Widening is exact; narrowing rounds to nearest even in hardware.
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 x = {a, b};
  bf16x2 y = __builtin_convertvector(x, bf16x2);
  return __builtin_bit_cast(uint32_t, y);
}
__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = bf_lo(u.x); f[1] = bf_hi(u.x); f[2] = bf_lo(u.y); f[3] = bf_hi(u.y);
  f[4] = bf_lo(u.z); f[5] = bf_hi(u.z); f[6] = bf_lo(u.w); f[7] = bf_hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  uint4 u;
  u.x = pack_bf16(f[0], f[1]); u.y = pack_bf16(f[2], f[3]);
  u.z = pack_bf16(f[4], f[5]); u.w = pack_bf16(f[6], f[7]);
  return u;
}

// Workgroups are dealt to the 8 XCDs (each with its own L2) round-robin by blockIdx.  This maps
// blockIdx to a logical id such that every XCD works through one contiguous run of logical ids
// (a bijection on [0, total) for any total): neighbouring query cubes, whose selected key cubes
// overlap when attention is local, then share an L2, and the XCDs work on different heads.
// Only for kernels whose workgroups all carry the same amount of work: a contiguous run of a
// list sorted by length would leave the XCDs unevenly loaded.
__device__ __forceinline__ unsigned xcd_chunked_id(unsigned b, unsigned total) {
  const unsigned x = b & 7u, per = total >> 3, rem = total & 7u;
  return x * per + (x < rem ? x : rem) + (b >> 3);
}

// x as bf16 hi + mid + lo (slots 0..2) and `slot3` as bf16 in slot 3 of an MFMA operand
__device__ __forceinline__ uint2 split3_bf16(float x, float slot3) {
  const __bf16 hi = (__bf16)x;
  const float r1 = x - (float)hi;
  const __bf16 mid = (__bf16)r1;
  const __bf16 lo = (__bf16)(r1 - (float)mid);
  auto bits = [](__bf16 v) { return (uint32_t)__builtin_bit_cast(unsigned short, v); };
  return make_uint2(bits(hi) | (bits(mid) << 16), bits(lo) | (bits((__bf16)slot3) << 16));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Validity mask of 64-row block `blk` (= cube blk / m, in-cube slots 64*(blk % m) .. +63): bit p is set
// iff in-cube slot s = 64*(blk % m) + p = (pt*Ch + ph)*Cw + pw holds a valid token.  Computed by a
// whole wavefront: lane p answers for bit p.
__device__ __forceinline__ uint64_t block_valid_mask_wave(const Geo& g, int blk, int lane) {
  const int c = blk / g.m, slot = (blk % g.m) * kTile + lane;
  const int cw = c % g.Nw, ch = (c / g.Nw) % g.Nh, ct = c / (g.Nw * g.Nh);
  const int pw = slot % g.Cw, ph = (slot / g.Cw) % g.Ch, pt = slot / (g.Cw * g.Ch);
  return __ballot(ct * g.Ct + pt < g.T && ch * g.Ch + ph < g.Hh && cw * g.Cw + pw < g.W);
}
// Valid tokens of the cube that block `blk` belongs to (the divisor of the pooled means).
__device__ __forceinline__ int cube_count(const uint64_t* __restrict__ mask, int blk, int m) {
  const int b0 = blk - blk % m;
  int n = 0;
  for (int s = 0; s < m; ++s) n += __popcll(mask[b0 + s]);
  return n;
}

}  // namespace vsa
