// Index rules of the block lists, shared by the kernels and by a host-side replay
// (vsa_host_replay_lists) so that the arithmetic that keeps every access inside its buffer can be
// checked on the CPU with hostile lists, without a GPU.
//
// A caller-supplied list (VSA_FLAG_INDICES_GIVEN) is not validated: entries outside [0, Nc),
// duplicates and disorder give unspecified VALUES, but no access may leave a buffer.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define VSA_RULE __host__ __device__ __forceinline__
#else
#define VSA_RULE inline
#endif

namespace vsa {

// Forward and dQ pass: the cube whose K/V tile is fetched for list entry `raw`.
VSA_RULE int clamp_cube(int raw, int ncubes) { return raw < 0 ? 0 : (raw > ncubes - 1 ? ncubes - 1 : raw); }

// Cubes of m blocks: entry u (0 <= u < m) of the block-level list that key cube `raw` expands to.
// Unsigned arithmetic, so that a hostile `raw` wraps around instead of overflowing; whatever comes
// out is clamped or skipped like any other entry.
VSA_RULE int expanded_entry(int raw, int m, int u) { return (int)((unsigned)raw * (unsigned)m + (unsigned)u); }

// Mismatched granularity: lists name tiles of (1,2,2) cubes.  Tile s = (st*Sh + sh)*Sw + sw (Sh = Nh/2,
// Sw = Nw/2) holds cubes (st, 2sh+a, 2sw+b); x = 2a + b in 0..3.  `s` is clamped first, so that a
// hostile entry still names a cube of the grid.
VSA_RULE int tile_member_cube(int s, int x, int Nt, int Nh, int Nw) {
  const int Sh = Nh / 2, Sw = Nw / 2, ns = Nt * Sh * Sw;
  s = s < 0 ? 0 : (s > ns - 1 ? ns - 1 : s);
  const int sw = s % Sw, sh = (s / Sw) % Sh, st = s / (Sw * Sh);
  return (st * Nh + 2 * sh + (x >> 1)) * Nw + 2 * sw + (x & 1);
}
// ... and the tile a cube belongs to
VSA_RULE int tile_of_cube(int c, int Nh, int Nw) {
  const int cw = c % Nw, ch = (c / Nw) % Nh, ct = c / (Nw * Nh);
  return (ct * (Nh / 2) + ch / 2) * (Nw / 2) + cw / 2;
}

// Key cubes of 16 tokens (Sec. 3.2, the 64 x 16 row of the tile-size tables): the (2,4,2) boxes inside a
// (4,4,4) cube.  Key cube 4*c + s, s = 2a + b, holds the in-cube slots (2a + tt)*16 + hh*4 + 2b + ww of
// cube c (tt, ww in {0,1}, hh in 0..3); its token x = tt*8 + hh*2 + ww sits at slot
// subcube_first_slot(s) + subcube_slot(x).
VSA_RULE int subcube_first_slot(int s) { return (s >> 1) * 32 + (s & 1) * 2; }
VSA_RULE int subcube_slot(int x) { return (x >> 3) * 16 + ((x >> 1) & 3) * 4 + (x & 1); }
// the in-cube slots of key cube s as a 64-bit pattern, and the 16 validity bits of its tokens (bit x =
// token x) out of the cube's 64-bit mask
VSA_RULE uint64_t subcube_pattern(int s) { return 0x33333333ull << (subcube_first_slot(s)); }
VSA_RULE uint32_t subcube_mask16(uint64_t cube_mask, int s) {
  uint32_t y = (uint32_t)(cube_mask >> subcube_first_slot(s)) & 0x33333333u;
  y = (y | (y >> 2)) & 0x0F0F0F0Fu;
  y = (y | (y >> 4)) & 0x00FF00FFu;
  y = (y | (y >> 8)) & 0x0000FFFFu;
  return y;
}

// Slot of the list read by lane `lane` for 64-entry chunk `chunk` of a list of n entries.
VSA_RULE int list_slot(int chunk, int lane, int n) {
  const int e = (chunk << 6) + lane;
  return e < n - 1 ? e : n - 1;
}

// Transposed map: an entry takes part iff it names a cube; a (query cube, key cube) pair is one
// bit, so duplicates collapse and a key cube's list never exceeds Nc entries, all lists of a
// (b, h) together never Nc * K.
VSA_RULE bool map_takes(int raw, int ncubes) { return (unsigned)raw < (unsigned)ncubes; }

// A transposed list of `deg` entries is worked off in split_runs(deg, seg) runs; run r covers the
// entries [run_bound(deg, runs, r), run_bound(deg, runs, r + 1)) of the list.
VSA_RULE int split_runs(int deg, int seg) { return deg > seg ? (deg + seg - 1) / seg : 1; }
VSA_RULE int run_bound(int deg, int runs, int r) { return (int)((long long)deg * r / runs); }
// Partial-result slots a list of `deg` entries wants at split length `seg` (none when it stays whole).
VSA_RULE int slots_wanted(int deg, int seg) { const int r = split_runs(deg, seg); return r > 1 ? r : 0; }
// The split length of a (b, h) is chosen so that all wanted slots fit; this is the guard behind it:
// a list gets its slots iff those wanted by the long lists before it (in cube order) plus its own
// stay within `cap`.
VSA_RULE bool split_granted(int runs, int wanted_before, int cap) { return runs > 1 && wanted_before + runs <= cap; }

}  // namespace vsa
