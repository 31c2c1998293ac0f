// Fine stage forward (Sec. 2.2 fine stage; Sec. 2.1 attention equation under the block mask)
// fused with the gated combine O = O_c * G_c + O_f * G_f.
//
// One workgroup (4 wavefronts) per (b, h, query cube).  The K selected key cubes are walked
// through a double-buffered LDS stage (K tile + V tile).  Work split inside the workgroup:
// wavefront (qh, kh) owns query rows qh*32..+31 and key rows kh*32..+31 of every key tile and
// keeps its OWN online-softmax state (running max, running sum, unnormalised O); the two
// key halves of a query row are merged once, after the last tile.  Splitting keys instead of
// queries halves the LDS traffic per MFMA (each K/V byte is read by two wavefronts, not four).
//
// Everything is computed transposed so that softmax statistics are per-lane scalars:
//   S^T[key, q]  = K_tile (A operand, row-major LDS reads) x Q^T (B operand, registers)
//   O^T[dv,  q] += V_tile^T (A operand, transposing LDS reads) x P^T (B operand = the S^T
//                  accumulator registers converted to bf16 in place)
// In the 32x32 accumulator layout lane l holds query column l%32 and 16 key (or dv) rows.
#include "fine_tile.h"
#include "vsa_kernels.h"

namespace vsa {

template <int D>
__global__ __launch_bounds__(256, 2) void k_fine_fwd(int Nc, int K, float sl2, const uint4* __restrict__ q,
                                                     const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                     const uint4* __restrict__ gc, const uint4* __restrict__ gf,
                                                     const int32_t* __restrict__ idx, const float* __restrict__ oc,
                                                     const uint64_t* __restrict__ mask, uint4* __restrict__ out,
                                                     uint4* __restrict__ out_fine, float* __restrict__ lse_f) {
  using TL = Tile<D>;
  constexpr int CPR = TL::CPR, KS = D / 16, DVB = D / 32, LPT = TL::LPT;
  constexpr int OS = D;  // fp32 row stride of the merge buffer
  constexpr int STAGE = 2 * TL::BYTES;  // K tile + V tile
  // Two separate LDS objects: the compiler can then tell that the asynchronous fill of one
  // stage does not alias the reads of the other and keeps the copy in flight during the math.
  __shared__ __attribute__((aligned(16))) unsigned char stage0[STAGE];
  __shared__ __attribute__((aligned(16))) unsigned char stage1[STAGE];
  __shared__ float ml[4 * 32 * 2];
  static_assert(2 * 32 * OS * 4 <= STAGE, "merge buffer must fit in one stage");

  const int c = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qh = wave & 1, kh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;  // first row of this (b,h)
  const int32_t* my_idx = idx + (bh * Nc + c) * (long long)K;

  int jt = my_idx[0];
  TL::async_load(k, rows0 + (long long)jt * kTile, stage0, wave, lane);
  TL::async_load(v, rows0 + (long long)jt * kTile, stage0 + TL::BYTES, wave, lane);

  bf16x8 qreg[KS];
  {
    const uint4* qrow = q + (rows0 + c * kTile + qh * 32 + l32) * CPR;
#pragma unroll
    for (int s = 0; s < KS; ++s) qreg[s] = __builtin_bit_cast(bf16x8, qrow[2 * s + h]);
  }

  float m2 = -INFINITY, lsum = 0.f;
  f32x16 o[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[x][i] = 0.f;
  __syncthreads();

  // One key tile: start the copy of the next tile pair into `nxt`, do the math on `cur`.
  auto body = [&](const unsigned char* cur, unsigned char* nxt, int t) {
    const uint64_t kmask = mask[jt];
    if (t + 1 < K) {
      jt = my_idx[t + 1];
      TL::async_load(k, rows0 + (long long)jt * kTile, nxt, wave, lane);
      TL::async_load(v, rows0 + (long long)jt * kTile, nxt + TL::BYTES, wave, lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char* Ks = cur;
    const unsigned char* Vs = cur + TL::BYTES;

    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) sacc = mfma32(TL::rowmajor_operand(Ks, kh * 32, s, lane), qreg[s], sacc);

    if (kmask != ~0ull) {  // pad keys of a partially filled cube never take part
      const uint32_t mh = (uint32_t)(kmask >> (kh * 32));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (!((mh >> (8 * (i / 4) + 4 * h + (i % 4))) & 1)) sacc[i] = -INFINITY;
    }

    float mx = sacc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sacc[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m2new = fmaxf(m2, mx * sl2);
    const float muse = (m2new == -INFINITY) ? 0.f : m2new;
    const float alpha = fast_exp2(m2 - muse);
    float p[16], rs = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = fast_exp2(fmaf(sacc[i], sl2, -muse));
      rs += p[i];
    }
    lsum = lsum * alpha + rs;
    m2 = m2new;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int x = 0; x < DVB; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[x][i] *= alpha;
    }
    const bf16x8 pb0 = acc_to_operand(p), pb1 = acc_to_operand(p + 8);
#pragma unroll
    for (int x = 0; x < DVB; ++x) {
      o[x] = mfma32(TL::transposed_operand(Vs, kh * 32, 0, x * 32, lane), pb0, o[x]);
      o[x] = mfma32(TL::transposed_operand(Vs, kh * 32, 1, x * 32, lane), pb1, o[x]);
    }
    __syncthreads();  // its fence also waits for this wave's share of the asynchronous copy
  };

  for (int t = 0; t < K; t += 2) {
    body(stage0, stage1, t);
    if (t + 1 < K) body(stage1, stage0, t + 1);
  }

  // ---- merge the two key halves, normalise, gate, store
  // Partial O of wave (qh, kh) goes to rows qh*32.. of stage `kh` (fp32 [64][D] each).
  lsum += __shfl_xor(lsum, 32);
  {
    float* Op = (float*)(kh == 0 ? stage0 : stage1) + qh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float4 val = make_float4(o[x][4 * g4], o[x][4 * g4 + 1], o[x][4 * g4 + 2], o[x][4 * g4 + 3]);
        *(float4*)&Op[l32 * OS + x * 32 + 8 * g4 + 4 * h] = val;
      }
  }
  if (h == 0) {
    ml[(wave * 32 + l32) * 2] = m2;
    ml[(wave * 32 + l32) * 2 + 1] = lsum;
  }
  __syncthreads();

  const uint64_t qmask = mask[c];
  const float* ocr = oc + (bh * Nc + c) * D;
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
    const int wa = r >> 5, wb = wa + 2, ql = r & 31;
    const float ma = ml[(wa * 32 + ql) * 2], la = ml[(wa * 32 + ql) * 2 + 1];
    const float mb = ml[(wb * 32 + ql) * 2], lb = ml[(wb * 32 + ql) * 2 + 1];
    const float M = fmaxf(ma, mb);
    float fa = fast_exp2(ma - M), fb = fast_exp2(mb - M);
    const float inv = 1.0f / (la * fa + lb * fb);
    fa *= inv; fb *= inv;
    const float* Oa = (const float*)stage0 + r * OS + ch * 8;
    const float* Ob = (const float*)stage1 + r * OS + ch * 8;
    float of[8], res[8];
    const float4 a0 = *(const float4*)Oa, a1 = *(const float4*)(Oa + 4);
    const float4 b0 = *(const float4*)Ob, b1 = *(const float4*)(Ob + 4);
    of[0] = a0.x * fa + b0.x * fb; of[1] = a0.y * fa + b0.y * fb; of[2] = a0.z * fa + b0.z * fb; of[3] = a0.w * fa + b0.w * fb;
    of[4] = a1.x * fa + b1.x * fb; of[5] = a1.y * fa + b1.y * fb; of[6] = a1.z * fa + b1.z * fb; of[7] = a1.w * fa + b1.w * fb;
    const long long g = (rows0 + c * kTile + r) * CPR + ch;
    const bool valid = (qmask >> r) & 1;
    uint4 ov = make_uint4(0, 0, 0, 0), fv = make_uint4(0, 0, 0, 0);
    if (valid) {
      float gcv[8], gfv[8];
      unpack8(gc[g], gcv);
      if (gf) unpack8(gf[g], gfv);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) gfv[e] = 1.f;
      }
      const float4 c0 = *(const float4*)(ocr + ch * 8), c1 = *(const float4*)(ocr + ch * 8 + 4);
      const float ocv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) res[e] = fmaf(ocv[e], gcv[e], of[e] * gfv[e]);
      ov = pack8(res);
      fv = pack8(of);
    }
    out[g] = ov;
    if (out_fine) out_fine[g] = fv;
  }
  if (lse_f && tid < kTile) {
    const int r = tid, wa = r >> 5, wb = wa + 2, ql = r & 31;
    const float ma = ml[(wa * 32 + ql) * 2], la = ml[(wa * 32 + ql) * 2 + 1];
    const float mb = ml[(wb * 32 + ql) * 2], lb = ml[(wb * 32 + ql) * 2 + 1];
    const float M = fmaxf(ma, mb);
    const float Lt = la * fast_exp2(ma - M) + lb * fast_exp2(mb - M);
    lse_f[rows0 + c * kTile + r] = ((qmask >> r) & 1) ? (M + fast_log2(Lt)) * kLn2 : 0.f;
  }
}

hipError_t launch_fine_fwd(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                           const void* gate_c, const void* gate_f, const int32_t* idx, const float* oc,
                           const uint64_t* mask, void* out, void* out_fine, float* lse_f, hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const unsigned grid = (unsigned)(BH * Nc);
  if (d == 128)
    k_fine_fwd<128><<<grid, 256, 0, s>>>(Nc, K, sl2, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                         (const uint4*)gate_c, (const uint4*)gate_f, idx, oc, mask, (uint4*)out,
                                         (uint4*)out_fine, lse_f);
  else
    k_fine_fwd<64><<<grid, 256, 0, s>>>(Nc, K, sl2, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                        (const uint4*)gate_c, (const uint4*)gate_f, idx, oc, mask, (uint4*)out,
                                        (uint4*)out_fine, lse_f);
  return hipGetLastError();
}

}  // namespace vsa
