// Token permutation (raster <-> cube-contiguous), cube validity masks and mean pooling.
// All three are pure data movement / fp32 adds: HBM-bandwidth bound, 16-byte accesses.
#include "list_rules.h"
#include "vsa_kernels.h"

namespace vsa {

// One workgroup per 64 destination rows of one (b, h).  The first wavefront works out, one row per
// lane, where each destination row comes from (the index arithmetic of the Sec. 2.2 equation, with
// its integer divisions, once per row instead of once per 16-byte chunk); then all 256 threads copy,
// several 16-byte chunks in flight per thread.
// Forward: destination = tiled row; its source is the raster row of the same (t,h,w), or zeros for
// a pad slot.  Inverse: destination = raster row.  H > 0: the raster tensor is [B, L, H, d]
// (token-major); H == 0: [B, H, L, d].
template <bool kInverse>
__global__ __launch_bounds__(256) void k_tile_permute(Geo g, int H, int chunks_per_row,
                                                      const uint4* __restrict__ src, uint4* __restrict__ dst) {
  __shared__ long long from[kTile], to[kTile];  // row numbers in units of rows; from < 0: a pad slot (zeros)
  const long long rows_dst = kInverse ? (long long)g.L : g.Np;
  const long long bh = blockIdx.y;
  const long long n0 = (long long)blockIdx.x * kTile;
  if (threadIdx.x < kTile) {
    const long long nn = n0 + threadIdx.x;
    long long f = -1, t_ = -1;
    if (nn < rows_dst) {
      const int n = (int)nn;
      if (!kInverse) {
        const int c = n / g.V, in = n % g.V;
        const int cw = c % g.Nw, chh = (c / g.Nw) % g.Nh, ct = c / (g.Nw * g.Nh);
        const int pw = in % g.Cw, ph = (in / g.Cw) % g.Ch, pt = in / (g.Cw * g.Ch);
        const int t = ct * g.Ct + pt, h = chh * g.Ch + ph, w = cw * g.Cw + pw;
        t_ = bh * g.Np + n;
        if (t < g.T && h < g.Hh && w < g.W) {
          const long long nr = ((long long)t * g.Hh + h) * g.W + w;
          f = H > 0 ? ((bh / H) * g.L + nr) * H + bh % H : bh * g.L + nr;
        }
      } else {
        const int w = n % g.W, h = (n / g.W) % g.Hh, t = n / (g.W * g.Hh);
        const long long c = ((long long)(t / g.Ct) * g.Nh + (h / g.Ch)) * g.Nw + (w / g.Cw);
        const int in = ((t % g.Ct) * g.Ch + (h % g.Ch)) * g.Cw + (w % g.Cw);
        t_ = H > 0 ? ((bh / H) * g.L + n) * H + bh % H : bh * g.L + n;
        f = bh * g.Np + c * g.V + in;
      }
    }
    from[threadIdx.x] = f;
    to[threadIdx.x] = t_;
  }
  __syncthreads();
  const int items = kTile * chunks_per_row;
  for (int i0 = 0; i0 < items; i0 += 4 * 256) {
    uint4 val[4];
    long long dsta[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int item = i0 + u * 256 + threadIdx.x, r = item / chunks_per_row, ch = item % chunks_per_row;
      dsta[u] = -1;
      val[u] = make_uint4(0, 0, 0, 0);
      if (item < items && to[r] >= 0) {
        dsta[u] = to[r] * chunks_per_row + ch;
        if (from[r] >= 0) val[u] = src[from[r] * chunks_per_row + ch];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (dsta[u] >= 0) dst[dsta[u]] = val[u];
  }
}

hipError_t launch_tile_permute(const Geo& g, int BH, int H_blhd, int d, const void* src, void* dst, bool inverse,
                               hipStream_t s) {
  const int cpr = d / 8;
  const long long rows_dst = inverse ? (long long)g.L : g.Np;
  dim3 grid((unsigned)((rows_dst + kTile - 1) / kTile), (unsigned)BH);
  if (inverse)
    k_tile_permute<true><<<grid, 256, 0, s>>>(g, H_blhd, cpr, (const uint4*)src, (uint4*)dst);
  else
    k_tile_permute<false><<<grid, 256, 0, s>>>(g, H_blhd, cpr, (const uint4*)src, (uint4*)dst);
  return hipGetLastError();
}

// Mean over the valid tokens of each cube (Sec. 2.2 coarse stage), fp32 result.
// One workgroup per (tensor, b*h, cube): V rows x D bf16 in (m blocks of 64 rows), D floats out.
// Thread t owns 16-byte chunk t % (D/8) of rows t / (D/8), t / (D/8) + 256/(D/8), ... of every
// block; the partial sums are added across row groups in a fixed order, so the result is
// deterministic.  The validity mask of each block comes from the geometry (one ballot per
// wavefront) and is also written to mask[block] for the kernels that follow (by the workgroups of
// the first (b, h) and tensor).
template <int D>
__global__ __launch_bounds__(256) void k_pool(Geo g, long long Np, uint64_t* __restrict__ mask,
                                              const uint4* __restrict__ q, const uint4* __restrict__ k,
                                              const uint4* __restrict__ v, float* __restrict__ qc,
                                              float* __restrict__ kc, float* __restrict__ vc) {
  constexpr int CPR = D / 8;        // chunks per row
  constexpr int RG = 256 / CPR;     // row groups
  constexpr int RPT = kTile / RG;   // rows per thread and block
  __shared__ float part[RG][D + 4];
  const int Nc = g.Nc;
  const int c = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const uint4* src = blockIdx.y == 0 ? q : (blockIdx.y == 1 ? k : v);
  float* dst = blockIdx.y == 0 ? qc : (blockIdx.y == 1 ? kc : vc);
  const int ch = threadIdx.x % CPR, rg = threadIdx.x / CPR;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int cnt = 0;
  for (int sb = 0; sb < g.m; ++sb) {
    const uint64_t m = block_valid_mask_wave(g, c * g.m + sb, threadIdx.x & 63);
    if (blockIdx.x < (unsigned)Nc && blockIdx.y == 0 && threadIdx.x == 0) mask[c * g.m + sb] = m;
    cnt += __popcll(m);
    const uint4* base = src + (bh * Np + ((long long)c * g.m + sb) * kTile) * CPR;
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      int r = rg + i * RG;
      uint4 u = base[r * CPR + ch];
      if ((m >> r) & 1) {
        float f[8];
        unpack8(u, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += f[e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][ch * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0;
    for (int r = 0; r < RG; ++r) s += part[r][threadIdx.x];
    dst[(bh * Nc + c) * D + threadIdx.x] = s / (float)cnt;
  }
}

// Key cubes of 16 tokens (Sec. 3.2, the 64 x 16 row of the tile-size tables): K and V are pooled over the
// four (2,4,2) boxes of every (4,4,4) cube, rows 4c .. 4c+3 of kc, vc.  One workgroup per (tensor, b*h,
// cube).  Thread (row group rg, chunk ch) adds rows rg, rg + RG, ...: of those, row r belongs to key
// cube 2a + b with a = r / 32 and b = (r / 2) % 2 = (rg / 2) % 2, so a thread keeps one partial sum per
// a, and key cube (a, b) is the sum over the row groups with that b, in ascending order.  A key cube
// without a valid token (a padded grid has them) gets zero rows and kcnt = 0: it is dead, left out of
// the coarse softmax and never selected.
template <int D>
__global__ __launch_bounds__(256) void k_pool_keys16(int Nc, int32_t* __restrict__ kcnt, const uint64_t* __restrict__ mask,
                                                     const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                     float* __restrict__ kc, float* __restrict__ vc) {
  constexpr int CPR = D / 8, RG = 256 / CPR, RPT = kTile / RG;
  static_assert(RG % 4 == 0 && 32 % RG == 0, "a thread's rows share b, and a changes between its rows only");
  __shared__ float part[2][RG][D + 4];
  const int c = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const uint4* src = blockIdx.y == 0 ? k : v;
  float* dst = blockIdx.y == 0 ? kc : vc;
  const int ch = threadIdx.x % CPR, rg = threadIdx.x / CPR;
  const uint64_t m = mask[c];
  float acc[2][8] = {{0, 0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0, 0}};
  const uint4* base = src + (bh * Nc + c) * (long long)kTile * CPR;
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg + i * RG;
    const uint4 u = base[r * CPR + ch];
    if ((m >> r) & 1) {
      float f[8];
      unpack8(u, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[(i * RG) >> 5][e] += f[e];  // = r / 32: rg < RG, and RG divides 32
    }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) part[a][rg][ch * 8 + e] = acc[a][e];
  __syncthreads();
  for (int o = threadIdx.x; o < 4 * D; o += 256) {
    const int sc = o / D, e = o % D, a = sc >> 1, b = sc & 1;
    const int cnt = __popcll(m & subcube_pattern(sc));
    float sum = 0;
    for (int r = 0; r < RG; ++r)
      if (((r >> 1) & 1) == b) sum += part[a][r][e];
    dst[((bh * Nc + c) * 4 + sc) * D + e] = cnt ? sum / (float)cnt : 0.f;
    if (e == 0 && bh == 0 && blockIdx.y == 0) kcnt[c * 4 + sc] = cnt;
  }
}

hipError_t launch_pool_keys16(int BH, int Nc, int d, const uint64_t* mask, int32_t* kcnt, const void* k, const void* v,
                              float* kc, float* vc, hipStream_t s) {
  dim3 grid((unsigned)(BH * Nc), 2);
  if (d == 128)
    k_pool_keys16<128><<<grid, 256, 0, s>>>(Nc, kcnt, mask, (const uint4*)k, (const uint4*)v, kc, vc);
  else
    k_pool_keys16<64><<<grid, 256, 0, s>>>(Nc, kcnt, mask, (const uint4*)k, (const uint4*)v, kc, vc);
  return hipGetLastError();
}

// tensors = 3: Q, K and V pooled per cube; tensors = 1: Q only (K and V are pooled by launch_pool_keys16)
hipError_t launch_pool(const Geo& g, int BH, int d, uint64_t* mask, const void* q, const void* k, const void* v,
                       float* qc, float* kc, float* vc, int tensors, hipStream_t s) {
  dim3 grid((unsigned)(BH * g.Nc), (unsigned)tensors);
  if (d == 128)
    k_pool<128><<<grid, 256, 0, s>>>(g, g.Np, mask, (const uint4*)q, (const uint4*)k, (const uint4*)v, qc, kc, vc);
  else
    k_pool<64><<<grid, 256, 0, s>>>(g, g.Np, mask, (const uint4*)q, (const uint4*)k, (const uint4*)v, qc, kc, vc);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Matrix-core rate probe for benchmarks: 4 wavefronts per workgroup, each running `iters` x 32
// v_mfma_f32_32x32x16_bf16 on 8 + 8 operands fetched once from `operands` (4 accumulators, 8-deep
// dependent chains, which the pipe runs at full rate).  No memory traffic inside the loop.
typedef __bf16 rate_bf16x8 __attribute__((ext_vector_type(8)));
typedef float rate_f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void k_mfma_rate(const uint4* __restrict__ operands, float* __restrict__ sink,
                                                   int iters) {
  rate_bf16x8 a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = __builtin_bit_cast(rate_bf16x8, operands[(threadIdx.x * 16 + j) & 4095]);
    b[j] = __builtin_bit_cast(rate_bf16x8, operands[(threadIdx.x * 16 + 8 + j) & 4095]);
  }
  rate_f32x16 c[4];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[x][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int j = 0; j < 8; ++j) c[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + x) & 7], c[x], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c[x][i];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_mfma_rate(const void* operands, float* sink, int workgroups, int iters, hipStream_t s) {
  k_mfma_rate<<<(unsigned)workgroups, 256, 0, s>>>((const uint4*)operands, sink, iters);
  return hipGetLastError();
}

}  // namespace vsa
