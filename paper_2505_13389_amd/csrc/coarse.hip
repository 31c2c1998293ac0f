// Coarse stage (Sec. 2.2): cube-level logits, softmax, O_c = A_c V_c, and the per-row top-K
// that turns a row of logits straight into an ascending block-index list (Sec. 2.4 fuses
// softmax, top-K and mask->index conversion in one kernel; so does k_coarse_rows below).
//
// Everything is fp32: the selection must agree with an fp32 reference except on near ties,
// and the whole stage is < 0.2 % of the attention FLOPs.  Three launches:
//   S  = scale * Qc Kc^T          fp32 matrix-core GEMM, S materialised [B*H, Nc, Nc]
//   k_coarse_rows                 one wavefront per row: log-sum-exp, top-K -> index list,
//                                 probabilities written back over S
//   Oc = P Vc                     fp32 matrix-core GEMM
#include "vsa_kernels.h"

namespace vsa {

__device__ __forceinline__ uint32_t sortable_key(float s) {
  uint32_t b = __float_as_uint(s);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// One wavefront per row of the score matrix; lane j holds logits j, j+64, ... (NCH per lane).
template <int NCH>
__global__ __launch_bounds__(256) void k_coarse_rows(int rows, int Nc, int K, float* __restrict__ sc,
                                                     float* __restrict__ lse_c, int32_t* __restrict__ idx,
                                                     int emit_idx) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  float* srow = sc + (long long)row * Nc;
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
  if (lane == 0 && lse_c) lse_c[row] = lse;

  if (emit_idx) {
    // K-th largest key by bitwise binary search: T = max{t : #(key >= t) >= K}, stopped early once a
    // prefix separates exactly K keys (the count is wave-uniform, so is the exit).
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = T | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        if (ch < nch) {
          uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[ch]) : 0u;
          cnt += __popcll(__ballot(key >= cand));
        }
      if (cnt >= K) {
        T = cand;
        if (cnt == K) break;  // exactly K keys at or above this prefix: the lower bits cannot change the set
      }
    }
    int n_gt = 0;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      if (ch < nch) {
        uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[ch]) : 0u;
        n_gt += __popcll(__ballot(key > T));
      }
    const int need = K - n_gt;  // entries equal to the threshold still to take, lowest index first
    int eq_seen = 0, base = 0;
    int32_t* out = idx + (long long)row * K;
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      if (ch < nch) {
        uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[ch]) : 0u;
        bool eq = (key == T) && (ch * 64 + lane < Nc);
        uint64_t beq = __ballot(eq);
        bool take = (key > T) || (eq && (eq_seen + __popcll(beq & lt) < need));
        eq_seen += __popcll(beq);
        uint64_t bsel = __ballot(take);
        if (take) out[base + __popcll(bsel & lt)] = ch * 64 + lane;
        base += __popcll(bsel);
      }
  }
}

hipError_t gemm32(int batch, int M, int N, int Kd, float alpha, const float* a, long long sab, int sam, int sak,
                  const float* b, long long sbb, int sbk, int sbn, float* c, long long scb, hipStream_t s);

hipError_t launch_coarse(int BH, int Nc, int d, int K, float scale, const float* qc, const float* kc, const float* vc,
                         float* sc, float* oc, float* lse_c, int32_t* idx, int emit_idx, hipStream_t s) {
  const long long sx = (long long)Nc * d, ss = (long long)Nc * Nc;
  hipError_t e;
  if ((e = gemm32(BH, Nc, Nc, d, scale, qc, sx, d, 1, kc, sx, 1, d, sc, ss, s)) != hipSuccess) return e;
  const int rows = BH * Nc;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  // NCH = logits per lane (compile-time bound of the per-lane loops): the smallest that covers Nc
  if (Nc <= 128)
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

}  // namespace vsa
