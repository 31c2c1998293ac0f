// LDS tile layout and MFMA operand access shared by the fine-stage kernels.
//
// A tile is 64 token rows x D bf16, row-major, stored in LDS WITHOUT padding; the 16-byte
// chunk c of row r lives at chunk position c ^ swz(r).  The swizzle is chosen so that both
// access patterns of the 32x32x16 MFMA operands are spread over distinct 16-byte bank groups:
//   - row-major reads (lane = row, same chunk): 16 consecutive rows hit 16 distinct slots;
//   - transposed reads (ds_read_b64_tr_b16: 4 consecutive rows x 64 contiguous bytes): the
//     4 rows land in 4 different 64-byte groups of the 256-byte bank line.
#pragma once
#include "list_rules.h"
#include "vsa_common.h"

namespace vsa {

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;

// Byte address of an LDS object inside the workgroup's LDS allocation.
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// 64 lanes x 16 bytes, global -> LDS at lds_addr + lane*16; `base` and `lds_addr` wave-uniform.
// M0 carries the LDS base of the instruction; it is written right before and named as clobbered.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "s"(lds_addr)
               : "memory", "m0");
}
// The same with an immediate byte offset, which the instruction adds to BOTH addresses (global and
// LDS): a run of copies whose LDS targets are IMM apart then shares one M0 value, the callers
// compensating in the per-lane global offsets.  0 <= IMM < 4096.
template <int IMM>
__device__ __forceinline__ void lds_dma16_at(const void* base, unsigned voff) {
  static_assert(IMM >= 0 && IMM < 4096, "13-bit signed instruction offset");
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(voff), "s"(base), "n"(IMM) : "memory");
}
// M0 is written here and read by the copies that follow in program order (volatile asm statements
// keep their order).  Nothing else in these kernels uses M0: no dynamically indexed register arrays
// (v_movrel), no GWS or message instructions.
__device__ __forceinline__ void set_m0(unsigned lds_addr) { asm volatile("s_mov_b32 m0, %0" : : "s"(lds_addr) : "m0", "memory"); }
__device__ __forceinline__ void lds_dma4(const void* base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(voff), "s"(base), "s"(lds_addr)
               : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
// A pointer the caller knows to be wave-uniform, forced into scalar registers.
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const unsigned long long a = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  return (const void*)(((unsigned long long)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// The list of key cubes a workgroup streams, with the valid-key mask of one 32-key half of each
// cube, held in registers 64 entries at a time (lane e holds entry e of the current chunk).  The
// loops read an entry with v_readlane: no scalar or vector load, and so no wait on one, sits
// between a barrier and the copies issued after it.  Entries must be visited in ascending order.
struct CubeList {
  const int32_t* list;
  const uint64_t* mask;
  int n, half, lane, chunk, idx_v, ncubes;
  uint32_t km_v;
  __device__ __forceinline__ void load_indices(int c) {
    chunk = c;
    idx_v = list[list_slot(c, lane, n)];
    asm volatile("" : "+v"(idx_v));  // consumed at once: the compiler's wait for the load is placed right here
    // a caller-supplied list is not trusted: an entry outside [0, ncubes) must not turn into an
    // out-of-bounds fetch (the result for such a list is unspecified, the access pattern is not)
    idx_v = clamp_cube(idx_v, ncubes);
  }
  __device__ __forceinline__ void load_masks() {
    const uint64_t m = mask[idx_v];
    km_v = half ? (uint32_t)(m >> 32) : (uint32_t)m;
  }
  __device__ __forceinline__ void load_chunk(int c) {
    load_indices(c);
    load_masks();
    asm volatile("" : "+v"(km_v));
  }
  // After init() the cube indices of the first chunk are there (cube() works); the key masks are
  // still in flight until the caller's next wait for its own loads, so that the first copies can
  // be issued one memory round trip earlier.
  __device__ __forceinline__ void init(const int32_t* list_, const uint64_t* mask_, int n_, int half_, int /*wave*/,
                                       int lane_, int ncubes_) {
    list = list_, mask = mask_, n = n_, half = half_, lane = lane_, ncubes = ncubes_;
    load_indices(0);
  }
  __device__ __forceinline__ int cube(int e) const { return __builtin_amdgcn_readlane(idx_v, e & 63); }
  // cube index and key mask of entry e (wave-uniform, 0 <= e < n)
  __device__ __forceinline__ void get(int e, int& cube, uint32_t& km) {
    if ((e >> 6) != chunk) load_chunk(e >> 6);
    cube = __builtin_amdgcn_readlane(idx_v, e & 63);
    km = (uint32_t)__builtin_amdgcn_readlane((int)km_v, e & 63);
  }
  // The walk in tiles (one tile = one list entry here): number of tiles, whether the list names every
  // cube, the first source row of this wave's share of tile t (valid after init for the first chunk),
  // and row + key mask of tile t.
  static constexpr int kEntriesPerTile = 1;
  __device__ __forceinline__ int tiles() const { return n; }
  __device__ __forceinline__ int first_row(int t) const { return cube(t) * kTile; }
  __device__ __forceinline__ void get_tile(int t, int& row, uint32_t& km) {
    int c;
    get(t, c, km);
    row = c * kTile;
  }
  template <class TL>
  __device__ static __forceinline__ void offsets(int wave, int lane, unsigned* off) { TL::lane_offsets(wave, lane, off); }
};

// Lists that name key cubes of 16 tokens (see subcube_* in list_rules.h): a streamed 64-key tile is
// gathered from four list entries, wavefront w copying the 16 rows of entry 4t + w into LDS rows
// 16w .. 16w+15 (a wave's copy instructions cover exactly those rows).  The per-lane source offsets
// are those of token order x inside a key cube, the key cube's first slot goes into the wave's base
// pointer.  Entries past the end of the list repeat the last one with an empty key mask.
struct SubCubeList {
  const int32_t* list;
  const uint64_t* mask;
  int n, half, wave, lane, chunk, idx_v, ncubes;
  uint32_t km_v;  // 16 validity bits of the lane's entry
  __device__ __forceinline__ void load_indices(int c) {
    chunk = c;
    idx_v = list[list_slot(c, lane, n)];
    asm volatile("" : "+v"(idx_v));
    idx_v = clamp_cube(idx_v, 4 * ncubes);  // (a caller-supplied list is not trusted)
  }
  __device__ __forceinline__ void load_masks() { km_v = subcube_mask16(mask[idx_v >> 2], idx_v & 3); }
  __device__ __forceinline__ void load_chunk(int c) {
    load_indices(c);
    load_masks();
    asm volatile("" : "+v"(km_v));
  }
  __device__ __forceinline__ void init(const int32_t* list_, const uint64_t* mask_, int n_, int half_, int wave_,
                                       int lane_, int ncubes_) {
    list = list_, mask = mask_, n = n_, half = half_, lane = lane_, ncubes = ncubes_;
    wave = __builtin_amdgcn_readfirstlane(wave_);
    load_indices(0);
  }
  static constexpr int kEntriesPerTile = 4;
  __device__ __forceinline__ int tiles() const { return (n + 3) >> 2; }
  __device__ __forceinline__ int row_of_entry(int e) const {  // e in the current chunk
    const int id = __builtin_amdgcn_readlane(idx_v, min(e, n - 1) & 63);
    return (id >> 2) * kTile + subcube_first_slot(id & 3);
  }
  __device__ __forceinline__ int first_row(int t) const { return row_of_entry(4 * t + wave); }
  __device__ __forceinline__ void get_tile(int t, int& row, uint32_t& km) {
    const int e0 = 4 * t;
    if ((e0 >> 6) != chunk) load_chunk(e0 >> 6);
    row = row_of_entry(e0 + wave);
    const int ea = e0 + 2 * half, eb = ea + 1;
    const uint32_t ma = (uint32_t)__builtin_amdgcn_readlane((int)km_v, ea & 63);
    const uint32_t mb = (uint32_t)__builtin_amdgcn_readlane((int)km_v, eb & 63);
    km = (ea < n ? ma : 0u) | ((eb < n ? mb : 0u) << 16);
  }
  template <class TL>
  __device__ static __forceinline__ void offsets(int wave, int lane, unsigned* off) { TL::lane_offsets_sub(wave, lane, off); }
};

template <int D>
struct Tile {
  static constexpr int CPR = D / 8;               // 16-byte chunks per row
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int BYTES = kTile * ROW_BYTES;
  static constexpr int LPT = kTile * CPR / 256;    // chunks per thread when 256 threads copy a tile

  __device__ static __forceinline__ int swz(int r) {
    if (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
  }
  __device__ static __forceinline__ int off(int r, int c) { return r * ROW_BYTES + ((c ^ swz(r)) << 4); }

  // 256 threads fetch one tile (rows row0..row0+63 of `src`, CPR chunks per row) into registers.
  __device__ static __forceinline__ void gload(const uint4* __restrict__ src, long long row0, int tid, uint4* regs) {
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
      int item = it * 256 + tid;
      regs[it] = src[(row0 + item / CPR) * CPR + item % CPR];
    }
  }
  __device__ static __forceinline__ void lstore(unsigned char* tile, int tid, const uint4* regs) {
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
      int item = it * 256 + tid;
      *(uint4*)(tile + off(item / CPR, item % CPR)) = regs[it];
    }
  }

  // Asynchronous global -> LDS copy of one tile by the 4 wavefronts of a workgroup, without
  // passing through registers (global_load_lds_dwordx4).  One wave instruction fills 1 KiB of
  // consecutive LDS (RPI rows); the swizzle is applied on the SOURCE side: the lane that writes
  // physical chunk pc of row r fetches logical chunk pc ^ swz(r).  The per-lane source offsets
  // do not depend on the tile and are computed once (lane_offsets); per tile the address is a
  // wave-uniform tile pointer (scalar registers) plus that 32-bit offset.
  //
  // The copy is issued from inline assembly on purpose: the compiler then keeps no record of it,
  // so it never drains it early, and the kernels order it by hand -- completion is counted by
  // vmcnt in issue order, every wave waits for its own share (s_waitcnt) and a workgroup barrier
  // then makes the whole tile visible.
  static constexpr int RPI = 1024 / ROW_BYTES;   // rows per wave instruction
  static constexpr int IPW = kTile / RPI / 4;    // instructions per wave and tile, 4 waves copying
  // NW wavefronts share the copy of one tile; `part` in [0, NW) is this wave's share.  The
  // offsets come out LESS the instruction offset (i KiB) that copy i of a tile carries: the
  // instruction adds its immediate to both the global and the LDS address, so one M0 value
  // serves all copies of a tile.  (The source row of copy i lies at least i KiB into the tile,
  // so the difference is never negative.)
  template <int NW = 4>
  __device__ static __forceinline__ void lane_offsets(int part, int lane, unsigned* off) {
    constexpr int N = kTile / RPI / NW;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int r = (part * N + i) * RPI + lane / CPR, pc = lane % CPR;
      off[i] = (unsigned)((r * CPR + (pc ^ swz(r))) * 16) - (unsigned)i * 1024u;
    }
  }
  // The same for a tile gathered from four key cubes of 16 tokens (SubCubeList), four wavefronts
  // copying: the base pointer of wave `part` is the first slot of its key cube, LDS row 16*part + x
  // takes token x of that key cube, and the swizzle follows the LDS row.
  __device__ static __forceinline__ void lane_offsets_sub(int part, int lane, unsigned* off) {
    constexpr int N = kTile / RPI / 4;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int x = i * RPI + lane / CPR, r = part * 16 + x, pc = lane % CPR;
      off[i] = (unsigned)((subcube_slot(x) * CPR + (pc ^ swz(r))) * 16) - (unsigned)i * 1024u;
    }
  }
  // copy i (compile-time) of this wave's share; M0 must hold the LDS address of the share
  template <int I>
  __device__ static __forceinline__ void copy_step(const void* g, const unsigned* off) {
    lds_dma16_at<I * 1024>(g, off[I]);
  }
  template <int NW = 4>
  __device__ static __forceinline__ void async_load(const uint4* __restrict__ src, long long row0, unsigned char* tile,
                                                    int part, const unsigned* off) {
    constexpr int N = kTile / RPI / NW;
    static_assert(N >= 1 && N <= 4, "copies per wave and tile");
    const void* g = uniform_ptr(src + row0 * CPR);
    set_m0(__builtin_amdgcn_readfirstlane(lds_address(tile) + (unsigned)(part * N) * 1024u));
    copy_step<0>(g, off);
    if (N > 1) copy_step<1 % N>(g, off);
    if (N > 2) copy_step<2 % N>(g, off);
    if (N > 3) copy_step<3 % N>(g, off);
  }

  // MFMA 32x32x16 operand whose 32-index is the tile ROW and whose contraction index runs
  // along D: lane l supplies tile[row0 + l%32][16*s + 8*(l/32) .. +7]  (one 16-byte read).
  __device__ static __forceinline__ bf16x8 rowmajor_operand(const unsigned char* tile, int row0, int s, int lane) {
    int r = row0 + (lane & 31);
    return *(const bf16x8*)(tile + off(r, 2 * s + (lane >> 5)));
  }

  // MFMA 32x32x16 operand whose 32-index runs along D (columns col0..col0+31) and whose
  // contraction index is the tile ROW, in the order the 32x32 accumulator layout produces:
  // for k-step s, lane half h = l/32 and j = 0..7 the row is row0 + 16*s + 8*(j/4) + 4*h + j%4.
  // Two transposing 8-byte LDS reads; in each 16-lane block, lanes 4e..4e+3 read row e.
  __device__ static __forceinline__ bf16x8 transposed_operand(const unsigned char* tile, int row0, int s, int col0,
                                                              int lane) {
    int L = lane & 15;
    int r1 = row0 + 16 * s + 4 * (lane >> 5) + (L >> 2);
    int col = col0 + ((lane >> 4) & 1) * 16 + 4 * (L & 3);
    int ch = col >> 3, sub = (col & 7) * 2;
    bf16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(tile + off(r1, ch) + sub));
    bf16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(tile + off(r1 + 8, ch) + sub));
    return __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
  }

  // The same two operand reads with the lane-dependent part of the address split off, for loops
  // that cannot afford one address register per read: the swizzle is an XOR on the chunk bits, so
  // the k-step s of a row-major operand and the column block x of a transposed operand enter as
  // an XOR with a constant, everything else as a constant byte offset.
  __device__ static __forceinline__ int rowmajor_lane(int row0, int lane) { return off(row0 + (lane & 31), lane >> 5); }
  __device__ static __forceinline__ bf16x8 rowmajor_at(const unsigned char* tile, int lane_part, int s) {
    return *(const bf16x8*)(tile + (lane_part ^ (s << 5)));
  }
  // valid for row0 a multiple of 32 (swz(r + 8) == swz(r) ^ 2 and swz(r + 16) == swz(r) then hold)
  __device__ static __forceinline__ void transposed_lane(int row0, int lane, int& b0, int& b1) {
    const int L = lane & 15;
    const int r1 = row0 + 4 * (lane >> 5) + (L >> 2);
    const int col = ((lane >> 4) & 1) * 16 + 4 * (L & 3);
    b0 = off(r1, col >> 3) + (col & 7) * 2;
    b1 = off(r1 + 8, col >> 3) + (col & 7) * 2;
  }
  __device__ static __forceinline__ bf16x8 transposed_at(const unsigned char* tile, int b0, int b1, int s, int x) {
    const unsigned char* p = tile + s * 16 * ROW_BYTES;
    bf16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + (b0 ^ (x << 6))));
    bf16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p + (b1 ^ (x << 6))));
    return __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
  }
};

// fp32 merge buffers [64][D] in LDS (partial results of the wavefronts that share output rows).
// A row is D*4 bytes, a multiple of the 256 bytes the 64 banks span, so the 32 lanes of an
// accumulator column (one row each) would all hit the same banks; the 16-byte chunks of a row are
// therefore XOR-ed with the row number (mod 16).  `col` is a multiple of 4.
__device__ __forceinline__ int merge_offset(int row, int col, int row_stride) {
  return row * row_stride + ((((col >> 2) ^ (row & 15)) << 2));
}

// fp32 accumulator values [8s .. 8s+7] -> bf16 operand of k-step s (see transposed_operand).
__device__ __forceinline__ bf16x8 acc_to_operand(const float* p) {
  uint4 u = pack8(p);
  return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

}  // namespace vsa
