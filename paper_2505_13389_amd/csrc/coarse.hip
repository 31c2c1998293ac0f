// Coarse stage (Sec. 2.2): cube-level logits, softmax, O_c = A_c V_c, and the per-row top-K
// that turns a row of logits straight into an ascending block-index list (Sec. 2.4 fuses
// softmax, top-K and mask->index conversion in one kernel; so does k_coarse_rows below).
//
// Everything is fp32: the selection must agree with an fp32 reference except on near ties,
// and the whole stage is < 0.2 % of the attention FLOPs.  One launch (k_coarse_fused, the faster
// form up to several hundred cubes) or three:
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
// `kcnt` (optional): valid tokens per key cube; a key cube with none is dead -- its logit counts as -inf,
// so it gets probability 0 and, K not exceeding the number of live key cubes, is never selected.
template <int NCH>
__device__ __forceinline__ void coarse_row(float* srow, int Nc, int K, float* lse_out, int32_t* out, int emit_idx,
                                           int lane, const int32_t* __restrict__ kcnt = nullptr) {
  const int nch = (Nc + 63) / 64;
  float s[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    const int j = ch * 64 + lane;
    s[ch] = (j < Nc && (!kcnt || kcnt[j] > 0)) ? srow[j] + 0.f : -INFINITY;
  }

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
        const bool take = (key[ch] > T) || (eq && (eq_seen + (int)__popcll(beq & lt) < need));
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
                                                     int emit_idx, const int32_t* __restrict__ kcnt) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  coarse_row<NCH>(sc + (long long)row * Nc, Nc, K, lse_c ? lse_c + row : nullptr, idx + (long long)row * K, emit_idx,
                  lane, kcnt);
}

// The whole coarse stage in ONE launch, the score block never leaving the chip (Sec. 2.4 fuses
// softmax, top-K and index conversion; App. D notes that the coarse stage weighs most at short
// sequences).  One workgroup of 16 wavefronts per (b, h, 16 query cubes) -- small blocks, so that even
// a short sequence gives every compute unit several workgroups -- with both operands of the two
// products read straight from L2 (Kc, Vc of a head are a few hundred KB):
//   1. logits: S[16 x Nc] = scale * Qc_block Kc^T with v_mfma_f32_16x16x4_f32 (fp32 products and
//      sums), one 16-column block per wavefront and round, into LDS;
//   2. one row per wavefront: log-sum-exp, top-K list, probabilities written back into LDS;
//   3. O_c block = P Vc, 16 columns per wavefront; the wavefronts left over split the contraction
//      and their partial sums are added in a fixed order through LDS.
// A 16x16x4 step contracts 4 values of k, k-group l/16 of lane l; with one 16-byte load per lane and
// operand (4 consecutive k) step j of four takes k = k0 + 4*(l/16) + j -- the same relabelling on
// both operands.  NCH*64 >= Nc bounds the row (and the LDS block: 16 x (NCH*64 + 4) floats).
typedef float f32x4m __attribute__((ext_vector_type(4)));
constexpr int kFusedMaxCubes = 1536;  // the LDS block of 16 rows: 98.6 KB at 1536 cubes
template <int D, int NCH>
__global__ __launch_bounds__(1024) void k_coarse_fused(int Nc, int K, float scale, const float* __restrict__ qc,
                                                       const float* __restrict__ kc, const float* __restrict__ vc,
                                                       float* __restrict__ oc, float* __restrict__ lse_c,
                                                       int32_t* __restrict__ idx, int emit_idx) {
  constexpr int R = 16;                  // query cubes per workgroup
  constexpr int LDS_ROW = NCH * 64 + 4;  // + 4: rows start 4 banks apart
  constexpr int QROW = D + 4;
  constexpr int CB = D / 16;             // 16-column blocks of O_c
  constexpr int KSPLIT = 16 / CB;        // wavefronts sharing one column block of O_c
  __shared__ __attribute__((aligned(16))) float S[R * LDS_ROW];
  __shared__ __attribute__((aligned(16))) float Qs[R * QROW];
  __shared__ __attribute__((aligned(16))) float part[16][64][4];
  const int blocks = (Nc + R - 1) / R;
  const int m0 = (blockIdx.x % blocks) * R;
  const long long bh = blockIdx.x / blocks;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;
  const float* kb = kc + bh * Nc * D;
  const float* vb = vc + bh * Nc * D;
  const int rows_valid = min(R, Nc - m0), kpad = (Nc + 15) & ~15;

  for (int i = tid; i < R * D; i += 1024) {
    const int r = i / D, e = i % D;
    Qs[r * QROW + e] = r < rows_valid ? qc[(bh * Nc + m0 + r) * D + e] : 0.f;
  }
  __syncthreads();
  // 1. logits (columns Nc .. kpad-1 are written as zero for the second product)
  for (int cb = wave; cb * 16 < kpad; cb += 16) {
    const int n = cb * 16 + l16;
    const float* krow = kb + (long long)min(n, Nc - 1) * D + 4 * kq;
    f32x4m acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k0 = 0; k0 < D; k0 += 16) {
      const float4 a = *(const float4*)&Qs[l16 * QROW + k0 + 4 * kq];
      const float4 b = *(const float4*)(krow + k0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) S[(4 * kq + i) * LDS_ROW + n] = n < Nc ? scale * acc[i] : 0.f;
  }
  __syncthreads();
  // 2. rows (rows of the block beyond Nc hold the logits of zero queries and are never stored)
  if (wave < rows_valid) {
    const long long row = bh * Nc + m0 + wave;
    coarse_row<NCH>(S + wave * LDS_ROW, Nc, K, lse_c ? lse_c + row : nullptr, idx + row * K, emit_idx, lane);
  }
  __syncthreads();
  // 3. O_c[m0 + m][e] = sum_n P[m][n] Vc[n][e]: wavefront (cb, ks) takes columns 16*cb.. and every
  //    KSPLIT-th group of 16 contraction values
  {
    const int cb = wave % CB, ks = wave / CB;
    f32x4m acc = {0.f, 0.f, 0.f, 0.f};
    const float* vcol = vb + cb * 16 + l16;
    for (int k0 = ks * 16; k0 < kpad; k0 += 16 * KSPLIT) {
      const float4 a = *(const float4*)&S[l16 * LDS_ROW + k0 + 4 * kq];
      const int kk = k0 + 4 * kq;
      float b[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = kk + j < Nc ? vcol[(long long)(kk + j) * D] : 0.f;
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b[0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b[1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b[2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b[3], acc, 0, 0, 0);
    }
    *(float4*)part[wave][lane] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    __syncthreads();
    if (ks == 0) {
      float4 sum = *(const float4*)part[wave][lane];
      for (int o = 1; o < KSPLIT; ++o) {
        const float4 x = *(const float4*)part[o * CB + cb][lane];
        sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
      }
      const float out[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m = 4 * kq + i;
        if (m < rows_valid) oc[(bh * Nc + m0 + m) * D + cb * 16 + l16] = out[i];
      }
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

// Nq query cubes against Nk key cubes (Nk = Nq, or 4 Nq with key cubes of 16 tokens, where `kcnt` marks
// the dead ones); sc is [BH,Nq,Nk].
hipError_t launch_coarse(int BH, int Nq, int Nk, int d, int K, float scale, const float* qc, const float* kc,
                         const float* vc, float* sc, float* oc, float* lse_c, int32_t* idx, int emit_idx, int fused,
                         const int32_t* kcnt, hipStream_t s) {
  const long long sq = (long long)Nq * d, sk = (long long)Nk * d, ss = (long long)Nq * Nk;
  hipError_t e;
  if (Nq == Nk && !kcnt && Nk <= kFusedMaxCubes && fused) {
    const int Nc = Nq;
    const unsigned fgrid = (unsigned)(BH * ((Nc + 15) / 16));
#define VSA_FUSED(NCH_)                                                                                             \
  do {                                                                                                              \
    if (d == 128) k_coarse_fused<128, NCH_><<<fgrid, 1024, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx); \
    else k_coarse_fused<64, NCH_><<<fgrid, 1024, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx);          \
  } while (0)
    // NCH = logits per lane of the row step: the smallest that covers Nc
    if (Nc <= 64) VSA_FUSED(1);
    else if (Nc <= 128) VSA_FUSED(2);
    else if (Nc <= 256) VSA_FUSED(4);
    else if (Nc <= 512) VSA_FUSED(8);
    else if (Nc <= 768) VSA_FUSED(12);
    else if (Nc <= 1024) VSA_FUSED(16);
    else VSA_FUSED(24);
#undef VSA_FUSED
    return hipGetLastError();
  }
  if ((e = gemm32(BH, Nq, Nk, d, scale, qc, sq, d, 1, kc, sk, 1, d, sc, ss, s)) != hipSuccess) return e;
  const int rows = BH * Nq;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  // NCH = logits per lane (compile-time bound of the per-lane loops): the smallest that covers Nk
#define VSA_ROWS(NCH_) k_coarse_rows<NCH_><<<grid, 256, 0, s>>>(rows, Nk, K, sc, lse_c, idx, emit_idx, kcnt)
  if (Nk <= 64) VSA_ROWS(1);
  else if (Nk <= 128) VSA_ROWS(2);
  else if (Nk <= 256) VSA_ROWS(4);
  else if (Nk <= 512) VSA_ROWS(8);
  else if (Nk <= 768) VSA_ROWS(12);
  else if (Nk <= 1024) VSA_ROWS(16);
  else if (Nk <= 1536) VSA_ROWS(24);
  else if (Nk <= 2560) VSA_ROWS(40);
  else VSA_ROWS(64);
#undef VSA_ROWS
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return gemm32(BH, Nq, d, Nk, 1.f, sc, ss, Nk, 1, vc, sk, d, 1, oc, sq, s);
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
  if (Ns <= 64) k_coarse_rows<1><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1, nullptr);
  else if (Ns <= 128) k_coarse_rows<2><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1, nullptr);
  else if (Ns <= 256) k_coarse_rows<4><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1, nullptr);
  else if (Ns <= 512) k_coarse_rows<8><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1, nullptr);
  else k_coarse_rows<16><<<grid, 256, 0, s>>>(rows, Ns, K, ps, nullptr, tile_idx, 1, nullptr);
  return hipGetLastError();
}

}  // namespace vsa
