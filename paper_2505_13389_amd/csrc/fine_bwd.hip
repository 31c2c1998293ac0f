// Fine stage backward (Sec. 2.4 states a backward kernel exists; this is FlashAttention-style
// recomputation of P from the saved log-sum-exp, on the block-sparse pattern):
//   P_ij = exp(S_ij - lse_i),  dP_ij = dOf_i . v_j,  dS_ij = P_ij (dP_ij - Delta_i)
//   dQ_i = scale sum_j dS_ij k_j      (query-tile-major pass over the index list)
//   dK_j = scale sum_i dS_ij q_i,  dV_j = sum_i P_ij dOf_i   (key-tile-major pass over the
//                                                             transposed block map)
// Both passes add the pooled-path gradient dXc[cube]/cnt to every valid row in their epilogue
// and write zeros to pad rows.  Work split and operand layouts follow the forward kernel: all
// products are computed transposed, the streamed tiles sit in a double-buffered LDS stage, the
// resident tile sits in registers, and each wavefront pair owning the same output rows is
// merged once at the end.
#include <type_traits>

#include "fine_tile.h"
#include "vsa_kernels.h"

namespace vsa {

// ---------------------------------------------------------------------------------------------
// dQ pass: one workgroup per (b, h, query cube); streams the K selected (K tile, V tile) pairs.
// Wavefront (qh, kh): query rows qh*32..+31, key rows kh*32..+31 of each tile.
template <int D>
__global__ __launch_bounds__(256, 2) void k_fine_bwd_dq(int Nc, int K, float sl2, float scale, const uint4* __restrict__ q,
                                                        const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                        const uint4* __restrict__ dof, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ ld,
                                                        const float* __restrict__ dqc, const uint64_t* __restrict__ mask,
                                                        uint4* __restrict__ dq) {
  using TL = Tile<D>;
  constexpr int CPR = TL::CPR, KS = D / 16, DVB = D / 32, LPT = TL::LPT;
  constexpr int OS = D;
  constexpr int STAGE = 2 * TL::BYTES;  // K tile + V tile
  __shared__ __attribute__((aligned(16))) unsigned char stage0[STAGE];
  __shared__ __attribute__((aligned(16))) unsigned char stage1[STAGE];
  static_assert(2 * 32 * OS * 4 <= STAGE, "merge buffer must fit in one stage");

  const int c = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qh = wave & 1, kh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;
  const int32_t* my_idx = idx + (bh * Nc + c) * (long long)K;
  const uint64_t qmask = mask[c];

  const long long qrow_g = rows0 + c * kTile + qh * 32 + l32;
  bf16x8 qreg[KS], doreg[KS];
  {
    const uint4* qrow = q + qrow_g * CPR;
    const uint4* dorow = dof + qrow_g * CPR;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qreg[s] = __builtin_bit_cast(bf16x8, qrow[2 * s + h]);
      doreg[s] = __builtin_bit_cast(bf16x8, dorow[2 * s + h]);
    }
  }
  // lse2 = lse*log2(e), +inf on pad query rows (then P = 0 and the row contributes nothing)
  float lse2 = ld[2 * qrow_g];
  float dl = ld[2 * qrow_g + 1];
  // Everything loaded the ordinary way must have arrived before the first hand-ordered copy is
  // issued (the compiler cannot see those copies; see Tile::async_load).
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qreg[s]), "+v"(doreg[s]));
  asm volatile("" : "+v"(lse2), "+v"(dl));

  unsigned goff[TL::IPW];
  TL::lane_offsets(wave, lane, goff);
  int jt = my_idx[0];
  TL::async_load(k, rows0 + (long long)jt * kTile, stage0, wave, goff);
  TL::async_load(v, rows0 + (long long)jt * kTile, stage0 + TL::BYTES, wave, goff);

  f32x16 acc[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[x][i] = 0.f;

  // Per tile: wait for this wave's share of tile t, barrier (tile t complete, and every wave is
  // done with tile t-1), start the copy of tile t+1 into the other stage, do the math on tile t.
  auto body = [&](const unsigned char* cur, unsigned char* nxt, int t) {
    const uint64_t kmask = mask[jt];
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (t + 1 < K) {
      jt = my_idx[t + 1];
      TL::async_load(k, rows0 + (long long)jt * kTile, nxt, wave, goff);
      TL::async_load(v, rows0 + (long long)jt * kTile, nxt + TL::BYTES, wave, goff);
    }
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char* Ks = cur;
    const unsigned char* Vs = cur + TL::BYTES;

    f32x16 sacc, dpacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
    for (int s = 0; s < KS; ++s) sacc = mfma32(TL::rowmajor_operand(Ks, kh * 32, s, lane), qreg[s], sacc);
#pragma unroll
    for (int s = 0; s < KS; ++s) dpacc = mfma32(TL::rowmajor_operand(Vs, kh * 32, s, lane), doreg[s], dpacc);

    float ds[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ds[i] = fast_exp2(fmaf(sacc[i], sl2, -lse2)) * (dpacc[i] - dl);
    if (kmask != ~0ull) {
      const uint32_t mh = (uint32_t)(kmask >> (kh * 32));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (!((mh >> (8 * (i / 4) + 4 * h + (i % 4))) & 1)) ds[i] = 0.f;
    }
    const bf16x8 b0 = acc_to_operand(ds), b1 = acc_to_operand(ds + 8);
#pragma unroll
    for (int x = 0; x < DVB; ++x) {
      acc[x] = mfma32(TL::transposed_operand(Ks, kh * 32, 0, x * 32, lane), b0, acc[x]);
      acc[x] = mfma32(TL::transposed_operand(Ks, kh * 32, 1, x * 32, lane), b1, acc[x]);
    }
  };

  for (int t = 0; t < K; t += 2) {
    body(stage0, stage1, t);
    if (t + 1 < K) body(stage1, stage0, t + 1);
  }
  __syncthreads();

  {
    float* Op = (float*)(kh == 0 ? stage0 : stage1) + qh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float4 val = make_float4(acc[x][4 * g4], acc[x][4 * g4 + 1], acc[x][4 * g4 + 2], acc[x][4 * g4 + 3]);
        *(float4*)&Op[l32 * OS + x * 32 + 8 * g4 + 4 * h] = val;
      }
  }
  __syncthreads();

  const float inv_cnt = 1.0f / (float)__popcll(qmask);
  const float* dqcr = dqc + (bh * Nc + c) * D;
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
    const float* Oa = (const float*)stage0 + r * OS + ch * 8;
    const float* Ob = (const float*)stage1 + r * OS + ch * 8;
    uint4 ov = make_uint4(0, 0, 0, 0);
    if ((qmask >> r) & 1) {
      float res[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) res[e] = fmaf(Oa[e] + Ob[e], scale, dqcr[ch * 8 + e] * inv_cnt);
      ov = pack8(res);
    }
    dq[(rows0 + c * kTile + r) * CPR + ch] = ov;
  }
}

hipError_t launch_fine_bwd_dq(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                              const void* dof, const int32_t* idx, const float* ld,
                              const float* dqc, const uint64_t* mask, void* dq, hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const unsigned grid = (unsigned)(BH * Nc);
  if (d == 128)
    k_fine_bwd_dq<128><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                            (const uint4*)dof, idx, ld, dqc, mask, (uint4*)dq);
  else
    k_fine_bwd_dq<64><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                           (const uint4*)dof, idx, ld, dqc, mask, (uint4*)dq);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// dK/dV pass: one workgroup per (b, h, key cube); streams the (Q tile, dOf tile) pairs of the
// query cubes that selected this key cube.  Wavefront (kh, qh): key rows kh*32..+31 (its output
// rows; K and V of those rows stay in registers), query rows qh*32..+31 of each streamed tile.
// Here S (not S^T) is formed, so a lane holds one key column and 16 query rows; the per-row pair
// (lse*log2 e, Delta) of the streamed query tile -- `ld`, written by the preprocess kernel with
// lse = +inf on pad rows so that pad queries give P = 0 -- is staged in LDS next to the tiles.
//
// One workgroup per CU (the whole register file for 4 wavefronts), four LDS stages, and the
// loop is software-pipelined inside each wavefront: iteration t forms S and dP of tile t+1
// (MFMA) while the exponentials of tile t run (VALU), then feeds P and dS of tile t to the
// dV / dK MFMAs.  Copies run three tiles ahead.  Per iteration: wait for this wave's share of
// tile t+1, one barrier (tile t+1 complete; every wave done with tile t-1), refill the stage of
// tile t-1 with tile t+3.  Past the end of the list the last tile is fetched again, so the
// number of copies in flight is the same in every iteration.
template <int D>
__global__ __launch_bounds__(256, 1) void k_fine_bwd_dkv(int Nc, int K, float sl2, float scale, const uint4* __restrict__ q,
                                                         const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                         const uint4* __restrict__ dof,
                                                         const int32_t* __restrict__ row_ptr,
                                                         const int32_t* __restrict__ col,
                                                         const float* __restrict__ ld,
                                                         const float* __restrict__ dkc, const float* __restrict__ dvc,
                                                         const uint64_t* __restrict__ mask, uint4* __restrict__ dk,
                                                         uint4* __restrict__ dv) {
  using TL = Tile<D>;
  constexpr int CPR = TL::CPR, KS = D / 16, DVB = D / 32, LPT = TL::LPT;
  constexpr int OS = D;
  constexpr int STAGE = 2 * TL::BYTES + 2 * kTile * 4;  // Q tile, dOf tile, (lse2, delta)[64]
  constexpr int NLP = 2 * TL::IPW + 1;                  // copies per wave and stage
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * STAGE];
  static_assert(2 * 64 * OS * 4 <= 4 * STAGE, "merge buffers must fit");

  const int j = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = wave & 1, qh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;
  const uint64_t kmask = mask[j];
  const int32_t* rp = row_ptr + bh * (Nc + 1);
  const int beg = rp[j], end = rp[j + 1];
  const int32_t* my_col = col + bh * (long long)Nc * K;

  bf16x8 kreg[KS], vreg[KS];
  {
    const uint4* krow = k + (rows0 + j * kTile + kh * 32 + l32) * CPR;
    const uint4* vrow = v + (rows0 + j * kTile + kh * 32 + l32) * CPR;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kreg[s] = __builtin_bit_cast(bf16x8, krow[2 * s + h]);
      vreg[s] = __builtin_bit_cast(bf16x8, vrow[2 * s + h]);
    }
  }
  const bool kvalid = (kmask >> (kh * 32 + l32)) & 1;
  // ordinary loads done before the first hand-ordered copy (see Tile::async_load)
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(kreg[s]), "+v"(vreg[s]));

  f32x16 dka[DVB], dva[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dka[x][i] = 0.f; dva[x][i] = 0.f; }

  if (beg < end) {
    unsigned goff[TL::IPW];
    TL::lane_offsets(wave, lane, goff);
    const unsigned lds0 = lds_address(smem);
    // fill stage `st` with the tiles of list entry min(t, end-1); every wave issues NLP copies
    auto fill = [&](int st, int t) {
      const int cq = __builtin_amdgcn_readfirstlane(my_col[min(t, end - 1)]);
      const long long r0 = rows0 + (long long)cq * kTile;
      unsigned char* sp = smem + st * STAGE;
      TL::async_load(q, r0, sp, wave, goff);
      TL::async_load(dof, r0, sp + TL::BYTES, wave, goff);
      if (lane < 8)  // 16 rows x (lse2, delta) = 128 bytes per wave
        lds_dma16(uniform_ptr(ld + 2 * r0), (unsigned)(wave * 128 + lane * 16),
                  __builtin_amdgcn_readfirstlane(lds0 + st * STAGE + 2 * TL::BYTES + wave * 128));
    };
    auto s_dp = [&](int st, f32x16& sacc, f32x16& dpacc) {  // S and dP of the tile in stage st
      const unsigned char* Qs = smem + st * STAGE;
      const unsigned char* Ds = Qs + TL::BYTES;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < KS; ++s) sacc = mfma32(TL::rowmajor_operand(Qs, qh * 32, s, lane), kreg[s], sacc);
#pragma unroll
      for (int s = 0; s < KS; ++s) dpacc = mfma32(TL::rowmajor_operand(Ds, qh * 32, s, lane), vreg[s], dpacc);
    };

    fill(0, beg);
    fill(1, beg + 1);
    fill(2, beg + 2);
    wait_vmcnt<2 * NLP>();
    __builtin_amdgcn_s_barrier();
    f32x16 sacc, dpacc;
    s_dp(0, sacc, dpacc);

    // ST = stage of tile t (tile t+1 sits in ST+1, tile t+3 goes where tile t-1 was)
    auto body = [&](auto st_tag, int t) {
      constexpr int ST = decltype(st_tag)::value;
      wait_vmcnt<NLP>();
      __builtin_amdgcn_s_barrier();
      fill((ST + 3) & 3, t + 3);
      __builtin_amdgcn_sched_barrier(0);
      const unsigned char* Qs = smem + ST * STAGE;
      const unsigned char* Ds = Qs + TL::BYTES;
      const float* ls = (const float*)(Qs + 2 * TL::BYTES);
      const unsigned char* Qn = smem + ((ST + 1) & 3) * STAGE;
      const unsigned char* Dn = Qn + TL::BYTES;

      // With one wavefront per SIMD nothing hides an LDS round trip, so every operand of the
      // iteration is requested up front, in the order it is consumed.
      bf16x8 qa[KS], da[KS], dt[DVB][2], qt[DVB][2];
      float4 la[4], lb[4];
#pragma unroll
      for (int s = 0; s < KS; ++s) qa[s] = TL::rowmajor_operand(Qn, qh * 32, s, lane);
#pragma unroll
      for (int s = 0; s < KS; ++s) da[s] = TL::rowmajor_operand(Dn, qh * 32, s, lane);
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        la[g4] = *(const float4*)&ls[2 * (qh * 32 + 8 * g4 + 4 * h)];
        lb[g4] = *(const float4*)&ls[2 * (qh * 32 + 8 * g4 + 4 * h) + 4];
      }
#pragma unroll
      for (int x = 0; x < DVB; ++x) {
        dt[x][0] = TL::transposed_operand(Ds, qh * 32, 0, x * 32, lane);
        dt[x][1] = TL::transposed_operand(Ds, qh * 32, 1, x * 32, lane);
      }
#pragma unroll
      for (int x = 0; x < DVB; ++x) {
        qt[x][0] = TL::transposed_operand(Qs, qh * 32, 0, x * 32, lane);
        qt[x][1] = TL::transposed_operand(Qs, qh * 32, 1, x * 32, lane);
      }
      __builtin_amdgcn_sched_barrier(0);

      // tile t+1: S, dP (independent of the arithmetic below, the scheduler interleaves them)
      f32x16 sn, dpn;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sn[i] = 0.f; dpn[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < KS; ++s) sn = mfma32(qa[s], kreg[s], sn);
#pragma unroll
      for (int s = 0; s < KS; ++s) dpn = mfma32(da[s], vreg[s], dpn);

      // tile t: P = exp2(S*sl2 - lse2), dS = P * (dP - Delta)
      float p[16], ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const float4 a = la[g4], b = lb[g4];
        const float lv[4] = {a.x, a.z, b.x, b.z}, dvv[4] = {a.y, a.w, b.y, b.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g4 + e;
          float pi = fast_exp2(fmaf(sacc[i], sl2, -lv[e]));
          if (!kvalid) pi = 0.f;
          p[i] = pi;
          ds[i] = pi * (dpacc[i] - dvv[e]);
        }
      }
      const bf16x8 pb0 = acc_to_operand(p), pb1 = acc_to_operand(p + 8);
      const bf16x8 sb0 = acc_to_operand(ds), sb1 = acc_to_operand(ds + 8);
#pragma unroll
      for (int x = 0; x < DVB; ++x) {
        dva[x] = mfma32(dt[x][0], pb0, dva[x]);
        dva[x] = mfma32(dt[x][1], pb1, dva[x]);
        dka[x] = mfma32(qt[x][0], sb0, dka[x]);
        dka[x] = mfma32(qt[x][1], sb1, dka[x]);
      }
      sacc = sn;
      dpacc = dpn;
    };

    for (int t = beg; t < end; t += 4) {
      body(std::integral_constant<int, 0>{}, t);
      if (t + 1 < end) body(std::integral_constant<int, 1>{}, t + 1);
      if (t + 2 < end) body(std::integral_constant<int, 2>{}, t + 2);
      if (t + 3 < end) body(std::integral_constant<int, 3>{}, t + 3);
    }
    wait_vmcnt<0>();  // the refetches issued past the end of the list
  }
  __syncthreads();

  // merge the two query halves; dK first, then dV through the same buffers
  const float inv_cnt = 1.0f / (float)__popcll(kmask);
  float* part0 = (float*)smem;
  float* part1 = (float*)smem + 64 * OS;
  for (int pass = 0; pass < 2; ++pass) {
    float* Op = (qh == 0 ? part0 : part1) + kh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x16& a = pass == 0 ? dka[x] : dva[x];
        float4 val = make_float4(a[4 * g4], a[4 * g4 + 1], a[4 * g4 + 2], a[4 * g4 + 3]);
        *(float4*)&Op[l32 * OS + x * 32 + 8 * g4 + 4 * h] = val;
      }
    __syncthreads();
    const float* pooled = (pass == 0 ? dkc : dvc) + (bh * Nc + j) * D;
    const float mul = pass == 0 ? scale : 1.0f;
    uint4* dst = pass == 0 ? dk : dv;
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
      const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
      const float* Oa = part0 + r * OS + ch * 8;
      const float* Ob = part1 + r * OS + ch * 8;
      uint4 ov = make_uint4(0, 0, 0, 0);
      if ((kmask >> r) & 1) {
        float res[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) res[e] = fmaf(Oa[e] + Ob[e], mul, pooled[ch * 8 + e] * inv_cnt);
        ov = pack8(res);
      }
      dst[(rows0 + j * kTile + r) * CPR + ch] = ov;
    }
    __syncthreads();
  }
}

hipError_t launch_fine_bwd_dkv(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                               const void* dof, const int32_t* row_ptr, const int32_t* col, const float* ld,
                               const float* dkc, const float* dvc, const uint64_t* mask, void* dk,
                               void* dv, hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const unsigned grid = (unsigned)(BH * Nc);
  if (d == 128)
    k_fine_bwd_dkv<128><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                             (const uint4*)dof, row_ptr, col, ld, dkc, dvc, mask, (uint4*)dk,
                                             (uint4*)dv);
  else
    k_fine_bwd_dkv<64><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v,
                                            (const uint4*)dof, row_ptr, col, ld, dkc, dvc, mask, (uint4*)dk,
                                            (uint4*)dv);
  return hipGetLastError();
}

}  // namespace vsa
