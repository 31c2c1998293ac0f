// Coarse stage (Sec. 2.2): cube-level logits, softmax, O_c = A_c V_c, and the per-row top-K
// that turns a row of logits straight into an ascending block-index list (Sec. 2.4 fuses
// softmax, top-K and mask->index conversion in one kernel; so does k_coarse_rows below).
//
// Everything is fp32: the selection must agree with an fp32 reference except on near ties,
// and the whole stage is < 0.2 % of the attention FLOPs.  Three launches (up to 256 cubes a
// single-launch form, k_coarse_fused, exists as well; it is the slower one on this chip):
//   S  = scale * Qc Kc^T          fp32 matrix-core GEMM, S materialised [B*H, Nc, Nc]
//   k_coarse_rows                 one wavefront per row: log-sum-exp, top-K -> index list,
//                                 probabilities written back over S
//   Oc = P Vc                     fp32 matrix-core GEMM
#include "gemm32_tile.h"
#include "list_rules.h"
#include "vsa_kernels.h"

namespace vsa {

__device__ __forceinline__ uint32_t sortable_key(float s) {
  uint32_t b = __float_as_uint(s);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// Reductions over the 64 lanes of a wavefront, result in every lane: four data-parallel-primitive
// steps inside each row of 16 lanes (quad swaps, half-row mirror, row mirror: register-to-register,
// no trip through the LDS permute path), then the four row results are combined through scalar
// registers.  The order of the additions is fixed.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce_bits(uint32_t x, Op op) {
  x = op(x, dpp_move<0xB1>(x));   // quad_perm [1,0,3,2]
  x = op(x, dpp_move<0x4E>(x));   // quad_perm [2,3,0,1]
  x = op(x, dpp_move<0x141>(x));  // row_half_mirror
  x = op(x, dpp_move<0x140>(x));  // row_mirror
  const uint32_t a = __builtin_amdgcn_readlane(x, 0), b = __builtin_amdgcn_readlane(x, 16);
  const uint32_t c = __builtin_amdgcn_readlane(x, 32), d = __builtin_amdgcn_readlane(x, 48);
  return op(op(a, b), op(c, d));
}
__device__ __forceinline__ float wave_max(float x) {
  return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t p, uint32_t q) {
    return __float_as_uint(fmaxf(__uint_as_float(p), __uint_as_float(q))); }));
}
__device__ __forceinline__ float wave_sum(float x) {
  return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t p, uint32_t q) {
    return __float_as_uint(__uint_as_float(p) + __uint_as_float(q)); }));
}
__device__ __forceinline__ uint32_t wave_umin(uint32_t x) { return wave_reduce_bits(x, [](uint32_t p, uint32_t q) { return min(p, q); }); }
__device__ __forceinline__ uint32_t wave_umax(uint32_t x) { return wave_reduce_bits(x, [](uint32_t p, uint32_t q) { return max(p, q); }); }

// One row of the score matrix worked off by one wavefront; lane j holds logits j, j+64, ... (NCH per
// lane).  `srow` may point into global memory or into LDS.  Writes the row's probabilities back over
// the logits, its log-sum-exp to *lse_out (if given) and, with emit_idx, the ascending list of its K
// largest logits (ties to the lower index) to `out`.
template <int NCH>
__device__ __forceinline__ void coarse_row(float* srow, int Nc, int K, float* lse_out, int32_t* out, int emit_idx,
                                           int lane) {
  const int nch = (Nc + 63) / 64;
  float s[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) s[ch] = (ch * 64 + lane < Nc) ? srow[ch * 64 + lane] + 0.f : -INFINITY;

  float m = -INFINITY;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) m = fmaxf(m, s[ch]);
  m = wave_max(m);
  float l = 0.f;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) l += fast_exp2((s[ch] - m) * kLog2e);
  l = wave_sum(l);
  const float lse = m + fast_log2(l) * kLn2;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch)
    if (ch * 64 + lane < Nc) srow[ch * 64 + lane] = fast_exp2((s[ch] - lse) * kLog2e);
  if (lane == 0 && lse_out) *lse_out = lse;

  if (emit_idx) {
    // Order-preserving integer keys; lanes beyond Nc hold key 0 and never count (every threshold
    // tried is >= 1).  T = the K-th largest key, by bisection of the key range [min, max]:
    // cnt(x) = #(key >= x) is non-increasing, cnt(lo) >= K > cnt(hi) throughout.  The search stops
    // as soon as a threshold separates exactly K keys (all counts are wave-uniform, so is the
    // exit): about log2(range / gap at rank K) steps on spread-out logits, 32 at most.
    uint32_t key[NCH];
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const bool valid = ch * 64 + lane < Nc;
      key[ch] = valid ? sortable_key(s[ch]) : 0u;
      if (valid) kmin = min(kmin, key[ch]);
      kmax = max(kmax, key[ch]);
    }
    kmin = wave_umin(kmin);
    kmax = wave_umax(kmax);
    auto count_ge = [&](uint32_t x) {
      int cnt = 0;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        if (ch < nch) cnt += __popcll(__ballot(key[ch] >= x));
      return cnt;
    };
    unsigned long long lo = kmin, hi = (unsigned long long)kmax + 1ull;
    uint32_t T = (uint32_t)lo;
    while (hi - lo > 1ull) {
      const uint32_t mid = (uint32_t)((lo + hi) >> 1);
      const int cnt = count_ge(mid);
      if (cnt >= K) {
        lo = mid;
        T = mid;
        if (cnt == K) break;  // exactly K keys at or above mid: they are the set
      } else {
        hi = mid;
      }
    }
    int n_gt = 0;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      if (ch < nch) n_gt += __popcll(__ballot(key[ch] > T));
    const int need = K - n_gt;  // entries equal to the threshold still to take, lowest index first
    int eq_seen = 0, base = 0;
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      if (ch < nch) {
        const bool eq = (key[ch] == T) && (ch * 64 + lane < Nc);
        const uint64_t beq = __ballot(eq);
        const bool take = (key[ch] > T) || (eq && (eq_seen + __popcll(beq & lt) < need));
        eq_seen += __popcll(beq);
        const uint64_t bsel = __ballot(take);
        const int pos = base + __popcll(bsel & lt);
        if (take && pos < K) out[pos] = ch * 64 + lane;  // (pos < K always holds for finite logits)
        base += __popcll(bsel);
      }
  }
}

template <int NCH>
__global__ __launch_bounds__(256) void k_coarse_rows(int rows, int Nc, int K, float* __restrict__ sc,
                                                     float* __restrict__ lse_c, int32_t* __restrict__ idx,
                                                     int emit_idx) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  coarse_row<NCH>(sc + (long long)row * Nc, Nc, K, lse_c ? lse_c + row : nullptr, idx + (long long)row * K, emit_idx,
                  lane);
}

// The whole coarse stage of a short sequence (Nc <= 256) in ONE launch, the score block never
// leaving the chip (Sec. 2.4 fuses softmax, top-K and index conversion; App. D notes that the coarse
// stage weighs most at short sequences).  One workgroup of 16 wavefronts per (b, h, 64 query cubes):
//   1. four teams of four wavefronts form the [64 x Nc] block of logits, 64 columns per team, with
//      fp32 matrix instructions into LDS;
//   2. the 16 wavefronts take the rows one by one (log-sum-exp, top-K list, probabilities written
//      back into LDS);
//   3. a second fp32 product of the probabilities with Vc gives the block's rows of O_c, 64 columns
//      per team.
// Same arithmetic, in the same order per element, as the three-launch path: bit-identical results.
constexpr int kFusedMaxCubes = 256;
template <int D, int NCH>
__global__ __launch_bounds__(1024) void k_coarse_fused(int Nc, int K, float scale, const float* __restrict__ qc,
                                                       const float* __restrict__ kc, const float* __restrict__ vc,
                                                       float* __restrict__ oc, float* __restrict__ lse_c,
                                                       int32_t* __restrict__ idx, int emit_idx) {
  constexpr int LDS_ROW = kFusedMaxCubes + 4;  // + 4: rows start 4 banks apart (conflict-free column reads)
  constexpr int TEAMS = 4;
  __shared__ __attribute__((aligned(16))) float S[64 * LDS_ROW];
  __shared__ __attribute__((aligned(16))) float As[TEAMS][64][36];
  __shared__ __attribute__((aligned(16))) float Bs[TEAMS][64][36];
  const int blocks = (Nc + 63) / 64;
  const int m0 = (blockIdx.x % blocks) * 64;
  const long long bh = blockIdx.x / blocks;
  const int team = threadIdx.x >> 8, tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const float* qb = qc + (bh * Nc + m0) * D;
  const float* kb = kc + bh * Nc * D;
  const float* vb = vc + bh * Nc * D;
  const int rows_valid = min(64, Nc - m0), kpad = (Nc + 31) & ~31;

  // 1. logits: S[m][n] = scale * Qc[m0 + m] . Kc[n]; columns Nc .. kpad-1 are zero for the second product
  {
    const int n0 = team * 64;
    f32x16g acc;
    gemm_tile_global(As[team], Bs[team], qb, D, 1, rows_valid, kb + (long long)min(n0, Nc - 1) * D, D, 1,
                     n0 < Nc ? Nc - n0 : 0, D, tid, acc);
    const int n = n0 + wn * 32 + l32;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = wm * 32 + 8 * (i / 4) + 4 * h + (i % 4);
      if (n < kpad) S[m * LDS_ROW + n] = n < Nc ? scale * acc[i] : 0.f;
    }
  }
  __syncthreads();
  // 2. rows: softmax statistics, top-K list, probabilities back into S (rows of the block beyond Nc
  //    hold the logits of zero queries and are never stored)
  for (int r = (int)(threadIdx.x >> 6); r < rows_valid; r += 16) {
    const long long row = bh * Nc + m0 + r;
    coarse_row<NCH>(S + r * LDS_ROW, Nc, K, lse_c ? lse_c + row : nullptr, idx + row * K, emit_idx, lane);
  }
  __syncthreads();
  // 3. O_c[m0 + m][e] = sum_n P[m][n] Vc[n][e]
  {
    const int e0 = team * 64;
    f32x16g acc;
    gemm_tile_lds_a(S, LDS_ROW, Bs[team], vb + min(e0, D - 1), 1, D, e0 < D ? D - e0 : 0, Nc, tid, acc);
    const int e = e0 + wn * 32 + l32;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = wm * 32 + 8 * (i / 4) + 4 * h + (i % 4);
      if (m < rows_valid && e < D) oc[(bh * Nc + m0 + m) * D + e] = acc[i];
    }
  }
}

hipError_t gemm32(int batch, int M, int N, int Kd, float alpha, const float* a, long long sab, int sam, int sak,
                  const float* b, long long sbb, int sbk, int sbn, float* c, long long scb, hipStream_t s);

// Cubes of m > 1 blocks (Sec. 3.2's larger tiles): the fine kernels work on 64-row blocks, so the
// list of key cubes of query cube c becomes, for each of the cube's m blocks, the list of the m
// blocks of every selected key cube (still ascending).  One thread per output entry.
__global__ __launch_bounds__(256) void k_expand_lists(long long total, int K, int m, const int32_t* __restrict__ idx,
                                                      int32_t* __restrict__ out) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;  // ((row * m + s) * K + t) * m + u
  if (e >= total) return;
  const int u = (int)(e % m);
  const long long t = (e / m) % K, row = e / ((long long)m * K * m);
  out[e] = expanded_entry(idx[row * K + t], m, u);
}
// Mismatched granularity (Sec. 3.2: coarse stage on cubes, fine stage on tiles of (1,2,2) cubes): the
// coarse attention map P [Nc x Nc] is averaged over the 2x2 cubes of the query tile and the 2x2
// cubes of the key tile; the top-K is then taken per row of the pooled map (k_coarse_rows).  One
// thread per pooled entry; the 16 terms are added in a fixed order (query cubes ascending, key cubes
// ascending within each), every term scaled by 1/16 first.
__global__ __launch_bounds__(256) void k_pool_scores(long long total, int Nt, int Nh, int Nw, const float* __restrict__ P,
                                                     float* __restrict__ Ps) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;  // (bh * Ns + sq) * Ns + sk
  if (e >= total) return;
  const int Nc = Nt * Nh * Nw, Ns = Nc / 4;
  const int sk = (int)(e % Ns), sq = (int)((e / Ns) % Ns);
  const long long bh = e / ((long long)Ns * Ns);
  const float* Pb = P + bh * Nc * Nc;
  float acc = 0.f;
#pragma unroll
  for (int xq = 0; xq < 4; ++xq) {
    const int c = tile_member_cube(sq, xq, Nt, Nh, Nw);
#pragma unroll
    for (int xk = 0; xk < 4; ++xk) acc += Pb[(long long)c * Nc + tile_member_cube(sk, xk, Nt, Nh, Nw)] * 0.0625f;
  }
  Ps[e] = acc;
}
// tile lists [BH,Ns,K] -> lists of 64-row blocks (= cubes) for every query cube, [BH,Nc,4K]
__global__ __launch_bounds__(256) void k_expand_tiles(long long total, int K, int Nt, int Nh, int Nw,
                                                      const int32_t* __restrict__ tile_idx, int32_t* __restrict__ out) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;  // ((bh * Nc + c) * K + t) * 4 + x
  if (e >= total) return;
  const int Nc = Nt * Nh * Nw, Ns = Nc / 4;
  const int x = (int)(e & 3), t = (int)((e >> 2) % K);
  const long long row = e / (4LL * K);
  const int c = (int)(row % Nc);
  const long long bh = row / Nc;
  out[e] = tile_member_cube(tile_idx[(bh * Ns + tile_of_cube(c, Nh, Nw)) * K + t], x, Nt, Nh, Nw);
}
hipError_t launch_expand_tiles(int BH, int Nt, int Nh, int Nw, int K, const int32_t* tile_idx, int32_t* idx_blocks,
                               hipStream_t s) {
  const long long total = (long long)BH * Nt * Nh * Nw * K * 4;
  k_expand_tiles<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(total, K, Nt, Nh, Nw, tile_idx, idx_blocks);
  return hipGetLastError();
}

hipError_t launch_expand_lists(int BH, int Nc, int K, int m, const int32_t* idx, int32_t* idx_blocks, hipStream_t s) {
  const long long total = (long long)BH * Nc * m * K * m;
  k_expand_lists<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(total, K, m, idx, idx_blocks);
  return hipGetLastError();
}

hipError_t launch_coarse(int BH, int Nc, int d, int K, float scale, const float* qc, const float* kc, const float* vc,
                         float* sc, float* oc, float* lse_c, int32_t* idx, int emit_idx, int fused, hipStream_t s) {
  const long long sx = (long long)Nc * d, ss = (long long)Nc * Nc;
  hipError_t e;
  if (Nc <= kFusedMaxCubes && fused) {
    const unsigned fgrid = (unsigned)(BH * ((Nc + 63) / 64));
#define VSA_FUSED(D_, NCH_) k_coarse_fused<D_, NCH_><<<fgrid, 1024, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx)
    // NCH = logits per lane of the row step: the smallest that covers Nc
    if (d == 128) {
      if (Nc <= 64) VSA_FUSED(128, 1); else if (Nc <= 128) VSA_FUSED(128, 2); else VSA_FUSED(128, 4);
    } else {
      if (Nc <= 64) VSA_FUSED(64, 1); else if (Nc <= 128) VSA_FUSED(64, 2); else VSA_FUSED(64, 4);
    }
#undef VSA_FUSED
    return hipGetLastError();
  }
  if ((e = gemm32(BH, Nc, Nc, d, scale, qc, sx, d, 1, kc, sx, 1, d, sc, ss, s)) != hipSuccess) return e;
  const int rows = BH * Nc;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  // NCH = logits per lane (compile-time bound of the per-lane loops): the smallest that covers Nc
  if (Nc <= 64)
    k_coarse_rows<1><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 128)
    k_coarse_rows<2><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 256)
    k_coarse_rows<4><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 512)
    k_coarse_rows<8><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 768)
    k_coarse_rows<12><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 1024)
    k_coarse_rows<16><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else if (Nc <= 1536)
    k_coarse_rows<24><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  else
    k_coarse_rows<64><<<grid, 256, 0, s>>>(rows, Nc, K, sc, lse_c, idx, emit_idx);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return gemm32(BH, Nc, d, Nc, 1.f, sc, ss, Nc, 1, vc, sx, d, 1, oc, sx, s);
}

// Top-K on the pooled coarse map: P [BH,Nc,Nc] (probabilities, as launch_coarse leaves them in its
// score buffer) -> pooled map `ps` [BH,Ns,Ns] -> ascending tile lists [BH,Ns,K].
hipError_t launch_pooled_select(int BH, int Nt, int Nh, int Nw, int K, const float* P, float* ps, int32_t* tile_idx,
                                hipStream_t s) {
  const int Ns = Nt * Nh * Nw / 4;
  const long long total = (long long)BH * Ns * Ns;
  k_pool_scores<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(total, Nt, Nh, Nw, P, ps);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rows = BH * Ns;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  if (Ns <= 64) k_coarse_rows<1><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1);
  else if (Ns <= 128) k_coarse_rows<2><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1);
  else if (Ns <= 256) k_coarse_rows<4><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1);
  else if (Ns <= 512) k_coarse_rows<8><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1);
  else k_coarse_rows<16><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1);
  return hipGetLastError();
}

}  // namespace vsa
