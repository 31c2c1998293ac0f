// 64x64 output tiles of an fp32 GEMM on the matrix cores, shared by the batched GEMM kernel and
// the single-launch coarse stage.
#pragma once
#include "vsa_common.h"

namespace vsa {

// Batched fp32 GEMM on the matrix cores (v_mfma_f32_32x32x2_f32: full fp32 products and sums),
// arbitrary strides:  C[b][m][n] = alpha * sum_k A(b,m,k) * B(b,k,n),
//   A(b,m,k) = a[b*sab + m*sam + k*sak],  B(b,k,n) = bm[b*sbb + k*sbk + n*sbn],  C row-major.
// Each operand must have one unit stride (k or the other axis).  64x64 output tile per workgroup,
// one 32x32 block per wavefront, 32-deep k slices staged in LDS as [row][k] (k contiguous) so a
// lane fetches 4 consecutive k of its row with one 16-byte read and feeds 4 MFMAs with it; the
// contraction index a lane half works on is k = 8j + 4h + e, the same for both operands.
// The summation order over k is fixed, so results are deterministic.
typedef float f32x16g __attribute__((ext_vector_type(16)));

// One thread's share of a 64-row x 32-k slice: 8 values.  sk == 1: 8 consecutive k of row tid/4;
// otherwise (rows contiguous in memory) 8 consecutive rows at k = tid/8, stored transposed.
// Out-of-range elements read as zero.  Fetch and store are separate so that the next slice can
// be in flight (in registers) while the matrix instructions work on the current one.
__device__ __forceinline__ void gemm_fetch(float* v, const float* __restrict__ base, int rows_valid, int k_valid,
                                           long long srow, long long sk, int tid) {
  if (sk == 1) {
    const int r = tid >> 2, kq = (tid & 3) * 8;
    const float* p = base + r * srow + kq;
    const bool vec = (r < rows_valid) && (kq + 8 <= k_valid) && ((srow & 3) == 0) && ((((uintptr_t)base) & 15) == 0);
    if (vec) {
      const float4 x = *(const float4*)p, y = *(const float4*)(p + 4);
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = (r < rows_valid && kq + i < k_valid) ? p[i] : 0.f;
    }
  } else {
    const int kk = tid >> 3, rq = (tid & 7) * 8;
    const float* p = base + (long long)kk * sk + (long long)rq * srow;
    const bool vec = (srow == 1) && (rq + 8 <= rows_valid) && (kk < k_valid) && ((sk & 3) == 0) &&
                     ((((uintptr_t)base) & 15) == 0);
    if (vec) {
      const float4 x = *(const float4*)p, y = *(const float4*)(p + 4);
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = (rq + i < rows_valid && kk < k_valid) ? p[i * srow] : 0.f;
    }
  }
}
__device__ __forceinline__ void gemm_store(float (*T)[36], const float* v, long long sk, int tid) {
  if (sk == 1) {
    const int r = tid >> 2, kq = (tid & 3) * 8;
    *(float4*)&T[r][kq] = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)&T[r][kq + 4] = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    const int kk = tid >> 3, rq = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) T[rq + i][kk] = v[i];
  }
}


// One 64x64 output tile, both operands staged from global memory: wave (wm, wn) = (wave & 1,
// wave >> 1) of the 256 threads ends up with its 32x32 block in `acc` (lane l: column l%32, rows
// 8*(i/4) + 4*(l/32) + i%4).  The next 32-deep slice is fetched into registers while the current one
// is multiplied.  Ends with a barrier: As, Bs may be reused at once.
// `tid` is the id within the 256 threads that share As, Bs.  A larger workgroup may run several such
// teams side by side, each with staging buffers of its own, as long as every team makes the same
// calls with the same Kd (the barriers are workgroup barriers); a team with nothing to compute
// passes m_valid or n_valid <= 0 (its operands then read as zero).
__device__ __forceinline__ void gemm_tile_global(float (*As)[36], float (*Bs)[36], const float* __restrict__ ab,
                                                 long long sam, long long sak, int m_valid,
                                                 const float* __restrict__ bb, long long sbn, long long sbk,
                                                 int n_valid, int Kd, int tid, f32x16g& acc) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1, l32 = lane & 31, h = lane >> 5;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  float va[8], vb[8];
  gemm_fetch(va, ab, m_valid, Kd, sam, sak, tid);
  gemm_fetch(vb, bb, n_valid, Kd, sbn, sbk, tid);
  for (int k0 = 0; k0 < Kd; k0 += 32) {
    gemm_store(As, va, sak, tid);
    gemm_store(Bs, vb, sbk, tid);
    __syncthreads();
    if (k0 + 32 < Kd) {  // next slice on its way while this one is multiplied
      gemm_fetch(va, ab + (long long)(k0 + 32) * sak, m_valid, Kd - k0 - 32, sam, sak, tid);
      gemm_fetch(vb, bb + (long long)(k0 + 32) * sbk, n_valid, Kd - k0 - 32, sbn, sbk, tid);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 av = *(const float4*)&As[wm * 32 + l32][8 * j + 4 * h];
      const float4 bv = *(const float4*)&Bs[wn * 32 + l32][8 * j + 4 * h];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc, 0, 0, 0);
    }
    __syncthreads();
  }
}

// The same with the A operand already in LDS: `a_lds` is a row-major [64][lda] fp32 block whose
// columns 0 .. Kd-1 (rounded up to a multiple of 32, the excess holding zeros) are the contraction
// axis.  Only B is staged.
__device__ __forceinline__ void gemm_tile_lds_a(const float* a_lds, int lda, float (*Bs)[36],
                                                const float* __restrict__ bb, long long sbn, long long sbk,
                                                int n_valid, int Kd, int tid, f32x16g& acc) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1, l32 = lane & 31, h = lane >> 5;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  float vb[8];
  gemm_fetch(vb, bb, n_valid, Kd, sbn, sbk, tid);
  const float* arow = a_lds + (wm * 32 + l32) * lda + 4 * h;
  for (int k0 = 0; k0 < Kd; k0 += 32) {
    gemm_store(Bs, vb, sbk, tid);
    __syncthreads();
    if (k0 + 32 < Kd) gemm_fetch(vb, bb + (long long)(k0 + 32) * sbk, n_valid, Kd - k0 - 32, sbn, sbk, tid);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 av = *(const float4*)(arow + k0 + 8 * j);
      const float4 bv = *(const float4*)&Bs[wn * 32 + l32][8 * j + 4 * h];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc, 0, 0, 0);
    }
    __syncthreads();
  }
}

}  // namespace vsa
