// Coarse stage (Sec. 2.2): cube-level logits, softmax, O_c = A_c V_c, and the per-row top-K
// that turns a row of logits straight into an ascending block-index list (Sec. 2.4: softmax,
// top-K and mask->index conversion in one kernel; here the logits never leave registers).
//
// Everything is fp32: the selection must agree with an fp32 reference except on near ties,
// and the whole stage is < 0.2 % of the attention FLOPs.
//
// One workgroup = 4 wavefronts = 4*RW query cubes of one (b,h).  Key cubes are streamed in
// chunks of 64 through LDS; lane j of a wavefront owns key cube chunk*64 + j of each of the
// wavefront's RW rows, so a row of Nc logits lives in Nc/64 registers per lane.
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

template <int D, int NCH, int RW>
__global__ __launch_bounds__(256) void k_coarse(int Nc, int K, float scale, const float* __restrict__ qc,
                                                const float* __restrict__ kc, const float* __restrict__ vc,
                                                float* __restrict__ oc, float* __restrict__ lse_c,
                                                int32_t* __restrict__ idx, int emit_idx) {
  constexpr int R = 4 * RW;   // rows per workgroup
  constexpr int KS = D + 4;   // LDS row stride of a staged chunk (floats): 16-byte reads, no bank conflicts
  __shared__ float qs[R][D];
  __shared__ float kbuf[64][KS];
  __shared__ float ps[R][NCH * 64];

  const int groups = (Nc + R - 1) / R;
  const int bh = blockIdx.x / groups;
  const int row0 = (blockIdx.x % groups) * R;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* qcb = qc + (long long)bh * Nc * D;
  const float* kcb = kc + (long long)bh * Nc * D;
  const float* vcb = vc + (long long)bh * Nc * D;
  const int nch = (Nc + 63) / 64;

  for (int i = threadIdx.x; i < R * D; i += 256) {
    int r = i / D, e = i % D;
    qs[r][e] = (row0 + r < Nc) ? qcb[(long long)(row0 + r) * D + e] : 0.f;
  }

  // ---- logits: s[r][ch] = scale * Qc[row] . Kc[ch*64 + lane]
  float s[RW][NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    if (ch < nch) {
      __syncthreads();
      for (int i = threadIdx.x; i < 64 * (D / 4); i += 256) {
        int j = i / (D / 4), e4 = i % (D / 4);
        int kj = ch * 64 + j;
        float4 val = make_float4(0, 0, 0, 0);
        if (kj < Nc) val = *(const float4*)(kcb + (long long)kj * D + e4 * 4);
        *(float4*)&kbuf[j][e4 * 4] = val;
      }
      __syncthreads();
      float acc[RW];
#pragma unroll
      for (int r = 0; r < RW; ++r) acc[r] = 0.f;
      for (int e4 = 0; e4 < D / 4; ++e4) {
        float4 kv = *(const float4*)&kbuf[lane][e4 * 4];
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          float4 qv = *(const float4*)&qs[wave * RW + r][e4 * 4];
          acc[r] = fmaf(qv.x, kv.x, acc[r]);
          acc[r] = fmaf(qv.y, kv.y, acc[r]);
          acc[r] = fmaf(qv.z, kv.z, acc[r]);
          acc[r] = fmaf(qv.w, kv.w, acc[r]);
        }
      }
#pragma unroll
      for (int r = 0; r < RW; ++r) s[r][ch] = (ch * 64 + lane < Nc) ? acc[r] * scale + 0.f : -INFINITY;
    } else {
#pragma unroll
      for (int r = 0; r < RW; ++r) s[r][ch] = -INFINITY;
    }
  }

  // ---- softmax statistics, probabilities to LDS, top-K
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int row = row0 + wave * RW + r;  // wave-uniform
    float m = -INFINITY;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) m = fmaxf(m, s[r][ch]);
    m = wave_max(m);
    float l = 0.f;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) l += fast_exp2((s[r][ch] - m) * kLog2e);
    l = wave_sum(l);
    const float lse = m + fast_log2(l) * kLn2;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch)
      if (ch < nch) ps[wave * RW + r][ch * 64 + lane] = fast_exp2((s[r][ch] - lse) * kLog2e);
    if (row < Nc && lane == 0 && lse_c) lse_c[(long long)bh * Nc + row] = lse;

    if (emit_idx && row < Nc) {
      // K-th largest key by bitwise binary search: T = max{t : #(key >= t) >= K}.
      uint32_t T = 0;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch)
          if (ch < nch) {
            uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[r][ch]) : 0u;
            cnt += __popcll(__ballot(key >= cand));
          }
        if (cnt >= K) T = cand;
      }
      int n_gt = 0;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        if (ch < nch) {
          uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[r][ch]) : 0u;
          n_gt += __popcll(__ballot(key > T));
        }
      const int need = K - n_gt;  // entries equal to the threshold still to take, lowest index first
      int eq_seen = 0, base = 0;
      int32_t* out = idx + ((long long)bh * Nc + row) * K;
      const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
        if (ch < nch) {
          uint32_t key = (ch * 64 + lane < Nc) ? sortable_key(s[r][ch]) : 0u;
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

  // ---- O_c = A_c V_c : lane owns output dims lane, lane+64; V chunks staged like the K chunks
  float o[RW][D / 64];
#pragma unroll
  for (int r = 0; r < RW; ++r)
#pragma unroll
    for (int x = 0; x < D / 64; ++x) o[r][x] = 0.f;
  for (int ch = 0; ch < nch; ++ch) {
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * (D / 4); i += 256) {
      int j = i / (D / 4), e4 = i % (D / 4);
      int kj = ch * 64 + j;
      float4 val = make_float4(0, 0, 0, 0);
      if (kj < Nc) val = *(const float4*)(vcb + (long long)kj * D + e4 * 4);
      *(float4*)&kbuf[j][e4 * 4] = val;
    }
    __syncthreads();
    const int jmax = min(64, Nc - ch * 64);
    for (int j4 = 0; j4 < jmax; j4 += 4) {
      float4 pv[RW];
#pragma unroll
      for (int r = 0; r < RW; ++r) pv[r] = *(const float4*)&ps[wave * RW + r][ch * 64 + j4];
#pragma unroll
      for (int x = 0; x < D / 64; ++x) {
        float v0 = kbuf[j4 + 0][lane + 64 * x], v1 = kbuf[j4 + 1][lane + 64 * x];
        float v2 = kbuf[j4 + 2][lane + 64 * x], v3 = kbuf[j4 + 3][lane + 64 * x];
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          o[r][x] = fmaf(pv[r].x, v0, o[r][x]);
          o[r][x] = fmaf(pv[r].y, v1, o[r][x]);
          o[r][x] = fmaf(pv[r].z, v2, o[r][x]);
          o[r][x] = fmaf(pv[r].w, v3, o[r][x]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int row = row0 + wave * RW + r;
    if (row < Nc)
#pragma unroll
      for (int x = 0; x < D / 64; ++x) oc[((long long)bh * Nc + row) * D + lane + 64 * x] = o[r][x];
  }
}

template <int D>
static hipError_t launch_coarse_d(int BH, int Nc, int K, float scale, const float* qc, const float* kc, const float* vc,
                                  float* oc, float* lse_c, int32_t* idx, int emit_idx, hipStream_t s) {
  if (Nc <= 512) {
    constexpr int RW = 2;
    k_coarse<D, 8, RW><<<BH * ((Nc + 4 * RW - 1) / (4 * RW)), 256, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx);
  } else if (Nc <= 1536) {
    constexpr int RW = 2;
    k_coarse<D, 24, RW><<<BH * ((Nc + 4 * RW - 1) / (4 * RW)), 256, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx);
  } else {
    constexpr int RW = 1;
    k_coarse<D, 64, RW><<<BH * ((Nc + 4 * RW - 1) / (4 * RW)), 256, 0, s>>>(Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx);
  }
  return hipGetLastError();
}

hipError_t launch_coarse(int BH, int Nc, int d, int K, float scale, const float* qc, const float* kc, const float* vc,
                         float* oc, float* lse_c, int32_t* idx, int emit_idx, hipStream_t s) {
  if (d == 128) return launch_coarse_d<128>(BH, Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx, s);
  return launch_coarse_d<64>(BH, Nc, K, scale, qc, kc, vc, oc, lse_c, idx, emit_idx, s);
}

}  // namespace vsa
