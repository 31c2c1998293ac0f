// Fine stage backward (Sec. 2.4 states a backward kernel exists; this is FlashAttention-style
// recomputation of P from the saved log-sum-exp, on the block-sparse pattern):
//   P_ij = exp(S_ij - lse_i),  dP_ij = dOf_i . v_j,  dS_ij = P_ij (dP_ij - Delta_i)
//   dQ_i = scale sum_j dS_ij k_j      (query-tile-major pass over the index list)
//   dK_j = scale sum_i dS_ij q_i,  dV_j = sum_i P_ij dOf_i   (key-tile-major pass over the
//                                                             transposed block map)
// Both passes add the pooled-path gradient dXc[cube]/cnt to every valid row in their epilogue
// and write zeros to pad rows.  Work split and operand layouts follow the forward kernel: the
// streamed tiles are copied global -> LDS asynchronously (two stages in the dQ pass, four in the
// dK/dV pass), the resident tile sits in registers, and each wavefront pair owning the same output
// rows is merged once at the end.  The per-row terms (lse, Delta) and the pad-key mask enter the
// products through extra MFMA steps rather than per-element vector arithmetic.
#include <type_traits>

#include "fine_tile.h"
#include "vsa_kernels.h"

namespace vsa {

// ---------------------------------------------------------------------------------------------
// dQ pass: one workgroup per (b, h, query cube); streams the K selected (K tile, V tile) pairs.
// Wavefront (qh, kh): query rows qh*32..+31, key rows kh*32..+31 of each tile.  LIST as in the forward
// kernel: one list entry per tile, or four key cubes of 16 tokens gathered into one.
template <int D, class LIST>
__global__ __launch_bounds__(256, 2) void k_fine_bwd_dq(int Nc, int K, float sl2, float scale, const uint4* __restrict__ q,
                                                        const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                        const uint4* __restrict__ dof, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ ld,
                                                        const float* __restrict__ dqc, const uint64_t* __restrict__ mask,
                                                        uint4* __restrict__ dq, int m_blocks) {
  using TL = Tile<D>;
  constexpr int CPR = TL::CPR, KS = D / 16, DVB = D / 32, LPT = TL::LPT;
  constexpr int OS = D;
  constexpr int STAGE = 2 * TL::BYTES;  // K tile + V tile
  __shared__ __attribute__((aligned(16))) unsigned char stage0[STAGE];
  __shared__ __attribute__((aligned(16))) unsigned char stage1[STAGE];
  static_assert(2 * 32 * OS * 4 <= STAGE, "merge buffer must fit in one stage");

  // (K = Nc: plain blockIdx order and staggered walks, as in the forward kernel)
  const int NT = (K + LIST::kEntriesPerTile - 1) / LIST::kEntriesPerTile;  // the walk is in tiles of 64 keys
  const bool same_lists = K == Nc * LIST::kEntriesPerTile;
  const unsigned wg = same_lists ? blockIdx.x : xcd_chunked_id(blockIdx.x, gridDim.x);
  const int c = wg % Nc;
  const long long bh = wg / Nc;
  const int rot = same_lists ? ((c >> 3) & 15) % NT : 0;
  auto ent = [&](int t) { const int e = t + rot; return e >= NT ? e - NT : e; };
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qh = wave & 1, kh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;
  const int32_t* my_idx = idx + (bh * Nc + c) * (long long)K;
  const uint64_t qmask = mask[c];

  // Start-up order: the list first (one round trip), then the copy of tile 0, and only then the
  // loads of the key masks, Q, dO_f and the per-row terms, so that everything the first iteration
  // needs is in flight together.  The empty asm consumes the loaded registers: the compiler has to
  // place its wait for them right there (it also drains the copy, which it cannot see), and its own
  // vmcnt bookkeeping has nothing left to wait for inside the loop (see Tile::async_load).
  unsigned goff[TL::IPW];
  LIST::template offsets<TL>(wave, lane, goff);
  LIST cubes;
  cubes.init(my_idx, mask, K, kh, wave, lane, Nc);
  {
    const int jt = cubes.first_row(ent(0));  // first source row of this wave's share
    TL::async_load(k, rows0 + jt, stage0, wave, goff);
    TL::async_load(v, rows0 + jt, stage0 + TL::BYTES, wave, goff);
  }
  cubes.load_masks();
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
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qreg[s]), "+v"(doreg[s]));
  asm volatile("" : "+v"(lse2), "+v"(dl), "+v"(cubes.km_v));
  uint32_t km_cur;  // valid-key mask (this wave's key half) of the tile of this iteration
  {
    int jt;
    cubes.get_tile(ent(0), jt, km_cur);
  }

  f32x16 acc[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[x][i] = 0.f;

  const int lane_a = TL::rowmajor_lane(kh * 32, lane);
  int lane_b0, lane_b1;
  TL::transposed_lane(kh * 32, lane, lane_b0, lane_b1);

  // Per-row terms folded into the matrix products (the vector pipe is the scarcer resource here):
  // one extra MFMA step adds -lse2[q]/sl2 to S^T, so that P = exp2(S' * sl2), plus a large negative
  // bias on pad keys; one extra step subtracts Delta[q] from dP^T.  Query-side operands (lane = query
  // column, slots 0..2 = the fp32 value split into three bf16 parts, slot 3 = 1 resp. 0) are fixed for
  // the workgroup; the key-side operand is (1, 1, 1, bias of key l%32).  Only the lane half h = 0
  // carries contraction slots 0..7; the other half is zero.  Pad query rows (lse = +inf) get a large
  // finite negative number: P underflows to exactly 0.
  constexpr uint32_t kOneBits = 0x3f80u, kBiasBits = 0xc6eau;  // bf16 1.0 and bf16(-29952)
  bf16x8 bq_s, bq_d, a_d;
  {
    const float inv_sl2 = 1.0f / sl2;
    const uint2 sb = split3_bf16(lse2 == INFINITY ? -30000.f : -lse2 * inv_sl2, 1.f), db = split3_bf16(-dl, 0.f);
    bq_s = __builtin_bit_cast(bf16x8, make_uint4(h == 0 ? sb.x : 0u, h == 0 ? sb.y : 0u, 0u, 0u));
    bq_d = __builtin_bit_cast(bf16x8, make_uint4(h == 0 ? db.x : 0u, h == 0 ? db.y : 0u, 0u, 0u));
    a_d = __builtin_bit_cast(bf16x8, make_uint4(h == 0 ? kOneBits * 0x10001u : 0u, h == 0 ? kOneBits : 0u, 0u, 0u));
  }

  // Per tile: wait for this wave's share of tile t, barrier (tile t complete, and every wave is
  // done with tile t-1), start the copy of tile t+1 into the other stage, do the math on tile t.
  auto body = [&](auto copy_tag, const unsigned char* cur, unsigned char* nxt, int t) {
    constexpr bool COPY = decltype(copy_tag)::value;  // false for the last tile of the list
    const uint32_t mh = km_cur;
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    // The copy of the next tile is not issued in one burst here -- eight wavefronts doing that at
    // the same moment queue up behind one another in the load path and stall -- but one
    // instruction per matrix step below.
    int jt = 0;
    if (COPY) cubes.get_tile(ent(t + 1), jt, km_cur);
    const void* gk = uniform_ptr(k + (rows0 + jt) * CPR);
    const void* gv = uniform_ptr(v + (rows0 + jt) * CPR);
    const unsigned ln = __builtin_amdgcn_readfirstlane(lds_address(nxt) + (unsigned)(wave * TL::IPW) * 1024u);
    auto copy_piece = [&](int i) {
      if (!COPY) return;
      if (i == 0) set_m0(ln);
      if (i == TL::IPW) set_m0(ln + TL::BYTES);
      if (i < 2 * TL::IPW) {
        const void* g = i < TL::IPW ? gk : gv;
        const int r = i % TL::IPW;
        if (r == 0) lds_dma16_at<0>(g, goff[0]);
        if (r == 1) lds_dma16_at<1024>(g, goff[1 % TL::IPW]);
        if (r == 2) lds_dma16_at<2048>(g, goff[2 % TL::IPW]);
        if (r == 3) lds_dma16_at<3072>(g, goff[3 % TL::IPW]);
      }
    };
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char* Ks = cur;
    const unsigned char* Vs = cur + TL::BYTES;

    // The LDS operands are requested a fixed number of matrix instructions ahead of their use, in
    // a pinned order (left to itself the compiler reads, waits and multiplies one operand at a
    // time).  Operand i: K rows (S^T steps), then V rows (dP^T steps), then transposed K (dQ^T
    // steps).  Operand addresses are rebuilt from three lane-dependent values (one XOR per read)
    // rather than held in registers across the loop: the register file is the scarce resource.
    int la = lane_a, lb0 = lane_b0, lb1 = lane_b1;
    asm volatile("" : "+v"(la), "+v"(lb0), "+v"(lb1));
    constexpr int NOP = 2 * KS + 2 * DVB, AHEAD = 4;
    bf16x8 op[NOP];
    auto read_op = [&](int i) {
      if (i < KS) return TL::rowmajor_at(Ks, la, i);
      if (i < 2 * KS) return TL::rowmajor_at(Vs, la, i - KS);
      const int j = i - 2 * KS;
      return TL::transposed_at(Ks, lb0, lb1, j & 1, j >> 1);
    };
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) op[i] = read_op(i);
    __builtin_amdgcn_sched_barrier(0);
    f32x16 sacc, dpacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i) {
      if (i < KS) sacc = mfma32(op[i], qreg[i < KS ? i : 0], sacc);
      else dpacc = mfma32(op[i], doreg[i < KS ? 0 : i - KS], dpacc);
      if (i + AHEAD < NOP) op[i + AHEAD] = read_op(i + AHEAD);
      if (!(i & 1)) copy_piece(i >> 1);
      __builtin_amdgcn_sched_barrier(0);
    }

    // one more step on each product brings in the per-row terms and the pad-key bias (see bq_s)
    {
      const bool dead = !((mh >> l32) & 1);
      const uint32_t w1 = kOneBits | ((dead ? kBiasBits : 0u) << 16);
      const bf16x8 a_s = __builtin_bit_cast(bf16x8, make_uint4(h == 0 ? kOneBits * 0x10001u : 0u, h == 0 ? w1 : 0u, 0u, 0u));
      sacc = mfma32(a_s, bq_s, sacc);
      dpacc = mfma32(a_d, bq_d, dpacc);
    }
    float ds[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ds[i] = fast_exp2(sacc[i] * sl2) * dpacc[i];
    const bf16x8 b0 = acc_to_operand(ds), b1 = acc_to_operand(ds + 8);
#pragma unroll
    for (int j = 0; j < 2 * DVB; ++j) {
      const int i = 2 * KS + j;
      acc[j >> 1] = mfma32(op[i], (j & 1) ? b1 : b0, acc[j >> 1]);
      if (i + AHEAD < NOP) op[i + AHEAD] = read_op(i + AHEAD);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  {
    const std::true_type copy;
    const std::false_type last;
    int t = 0;
    for (; t + 2 < NT; t += 2) {
      body(copy, stage0, stage1, t);
      body(copy, stage1, stage0, t + 1);
    }
    if (t + 1 < NT) {
      body(copy, stage0, stage1, t);
      body(last, stage1, stage0, t + 1);
    } else {
      body(last, stage0, stage1, t);
    }
  }
  // the pooled-gradient term of this thread's column chunk (the same chunk for all of its items),
  // requested before the partial results go through LDS
  static_assert(256 % CPR == 0, "a thread keeps its column chunk");
  const float* dqcr = dqc + ((bh * Nc + c) / m_blocks) * D + (tid % CPR) * 8;  // per cube = m_blocks blocks
  const float4 pc0 = *(const float4*)dqcr, pc1 = *(const float4*)(dqcr + 4);
  __syncthreads();

  {
    float* Op = (float*)(kh == 0 ? stage0 : stage1) + qh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float4 val = make_float4(acc[x][4 * g4], acc[x][4 * g4 + 1], acc[x][4 * g4 + 2], acc[x][4 * g4 + 3]);
        *(float4*)&Op[merge_offset(l32, x * 32 + 8 * g4 + 4 * h, OS)] = val;
      }
  }
  __syncthreads();

  const float inv_cnt = 1.0f / (float)cube_count(mask, c, m_blocks);
  const float pooled[8] = {pc0.x * inv_cnt, pc0.y * inv_cnt, pc0.z * inv_cnt, pc0.w * inv_cnt,
                           pc1.x * inv_cnt, pc1.y * inv_cnt, pc1.z * inv_cnt, pc1.w * inv_cnt};
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
    const int m0 = merge_offset(r, ch * 8, OS), m1 = merge_offset(r, ch * 8 + 4, OS);
    const float4 a0 = *(const float4*)((const float*)stage0 + m0), a1 = *(const float4*)((const float*)stage0 + m1);
    const float4 b0 = *(const float4*)((const float*)stage1 + m0), b1 = *(const float4*)((const float*)stage1 + m1);
    const float sum[8] = {a0.x + b0.x, a0.y + b0.y, a0.z + b0.z, a0.w + b0.w, a1.x + b1.x, a1.y + b1.y, a1.z + b1.z, a1.w + b1.w};
    uint4 ov = make_uint4(0, 0, 0, 0);
    if ((qmask >> r) & 1) {
      float res[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) res[e] = fmaf(sum[e], scale, pooled[e]);
      ov = pack8(res);
    }
    dq[(rows0 + c * kTile + r) * CPR + ch] = ov;
  }
}

hipError_t launch_fine_bwd_dq(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                              const void* dof, const int32_t* idx, const float* ld,
                              const float* dqc, const uint64_t* mask, void* dq, int m_blocks, int key_cubes_16,
                              hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const unsigned grid = (unsigned)(BH * Nc);
#define VSA_DQ(D_, LIST_)                                                                                          \
  k_fine_bwd_dq<D_, LIST_><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v, \
                                                (const uint4*)dof, idx, ld, dqc, mask, (uint4*)dq, m_blocks)
  if (key_cubes_16) {  // K counts key cubes of 16 tokens
    if (d == 128) VSA_DQ(128, SubCubeList);
    else VSA_DQ(64, SubCubeList);
  } else {
    if (d == 128) VSA_DQ(128, CubeList);
    else VSA_DQ(64, CubeList);
  }
#undef VSA_DQ
  return hipGetLastError();
}

// Key cubes of 16 tokens: the pooled-gradient term of row r of a key block, chunk ch -- the pooled
// gradient of the row's key cube (rows 4*block .. 4*block+3 of `pooled`) over the cube's valid tokens.
__device__ __forceinline__ void subcube_pooled_term(const float* __restrict__ pooled, long long first_row, uint64_t kmask,
                                                    int r, int D, int ch, float* out) {
  const int sc = 2 * (r >> 5) + ((r >> 1) & 1);
  const float inv = 1.0f / (float)__popcll(kmask & subcube_pattern(sc));  // (row r is valid: at least 1)
  const float* p = pooled + (first_row + sc) * D + ch * 8;
  const float4 p0 = *(const float4*)p, p1 = *(const float4*)(p + 4);
  out[0] = p0.x * inv; out[1] = p0.y * inv; out[2] = p0.z * inv; out[3] = p0.w * inv;
  out[4] = p1.x * inv; out[5] = p1.y * inv; out[6] = p1.z * inv; out[7] = p1.w * inv;
}

// ---------------------------------------------------------------------------------------------
// dK/dV pass: one workgroup per (b, h, key cube); streams the (Q tile, dOf tile) pairs of the
// query cubes that selected this key cube.  Wavefront (kh, qh): key rows kh*32..+31 (its output
// rows; K and V of those rows stay in registers), query rows qh*32..+31 of each streamed tile.
// Here S (not S^T) is formed, so a lane holds one key column and 16 query rows.  The per-row pair
// (lse*log2 e, Delta) of the streamed query tile -- `ld`, written by the preprocess kernel with
// lse = +inf on pad rows so that pad queries give P = 0 -- is staged in LDS next to the tiles and
// enters S and dP through one extra MFMA step each (split into three bf16 parts), as does the
// large negative bias of pad keys.
//
// One workgroup per CU (the whole register file for 4 wavefronts) and four LDS stages.  With a
// single wavefront per SIMD nothing but the wavefront's own instruction order overlaps the matrix
// pipe with LDS reads, copies and vector arithmetic, so the loop body is one basic block whose
// order is pinned by scheduling barriers: every step is one MFMA plus its share of the other
// work.  The loop is software-pipelined over three tiles: iteration t issues dV, dK of tile t,
// turns S', dP' of tile t+1 into P, dS, and forms S', dP' of tile t+2; the LDS operands of each
// phase are read during the phase before it.  Copies run four tiles ahead (two iterations of
// flight).  Per iteration: wait for this wave's share of tile t+2, one barrier (tile t+2
// complete; every wave done reading tile t), refill the stage of tile t with tile t+4.  Past the
// end of the list the last tile is fetched again, so the number of copies in flight is the same
// in every iteration.
//
// SUB: the lists name key cubes of 16 tokens (Sec. 3.2, the 64 x 16 row of the tile-size tables).  The
// workgroup still owns a 64-row key block; its list is the union of the lists of the block's four key
// cubes, and every entry says (bits 16..19) which of them the query block selected: the other key rows
// get the pad-key bias for that tile.  The pooled-gradient terms are per key cube.
template <int D, bool SUB>
__global__ __launch_bounds__(256, 1) void k_fine_bwd_dkv(int Nc, int K, float sl2, float scale, const uint4* __restrict__ q,
                                                         const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                         const uint4* __restrict__ dof,
                                                         const int32_t* __restrict__ col,
                                                         const int32_t* __restrict__ order, int items_per_bh,
                                                         float* __restrict__ parts, int cap,
                                                         const uint4* __restrict__ ldb,
                                                         const float* __restrict__ dkc, const float* __restrict__ dvc,
                                                         const uint64_t* __restrict__ mask, uint4* __restrict__ dk,
                                                         uint4* __restrict__ dv, int m_blocks) {
  using TL = Tile<D>;
  constexpr int CPR = TL::CPR, KS = D / 16, DVB = D / 32, LPT = TL::LPT;
  constexpr int OS = D;
  constexpr int STAGE = 2 * TL::BYTES + kTile * 16;  // Q tile, dOf tile, 16 bytes of (lse2, Delta) operand slots per row
  constexpr int NLP = 2 * TL::IPW + 1;                  // copies per wave and stage
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * STAGE];

  // Start-up: one descriptor load (key cube, begin and end of its run of the cube's list, slot; the
  // items of a (b, h) come longest first), then the list chunk, the key mask and the resident K, V
  // rows all in flight together, one wait, then the first copies.  A list longer than the split
  // length is shared by several workgroups, each of which leaves its fp32 partial sums in its slot
  // (desc.w >= 0) for k_dkv_reduce; unused descriptors carry key cube -1.
  const long long bh = blockIdx.x / items_per_bh;
  const int4 desc = ((const int4*)order)[blockIdx.x];
  if (desc.x < 0) return;
  const int j = desc.x, beg = desc.y, end = desc.z, n = end - beg, slot = desc.w;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = wave & 1, qh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;
  const int32_t* my_col = col + bh * (long long)Nc * K;
  // The list of streamed query cubes sits in a register, 64 entries at a time (lane e holds
  // entry e of the current chunk), so that the loop reads an index with v_readlane and issues
  // no scalar or vector memory load of its own.
  int chunk = 0;
  int col_v = n > 0 ? my_col[beg + list_slot(0, lane, n)] : 0;
  const uint64_t kmask = mask[j];

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
  asm volatile("" : "+v"(col_v));

  f32x16 dka[DVB], dva[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dka[x][i] = 0.f; dva[x][i] = 0.f; }

  if (beg < end) {
    unsigned goff[TL::IPW];
    TL::lane_offsets(wave, lane, goff);
    const unsigned lds0 = lds_address(smem);
    auto entry = [&](int t) {  // list entry min(t, end - 1): the query block (SUB: and the selected key cubes above it)
      const int e = min(t, end - 1) - beg;
      if ((e >> 6) != chunk) {
        chunk = e >> 6;
        col_v = my_col[beg + list_slot(chunk, lane, n)];
        asm volatile("" : "+v"(col_v));  // its wait stays inside this branch
      }
      return __builtin_amdgcn_readlane(col_v, e & 63);
    };
    // fill stage `st` with the tiles of list entry min(t, end-1); every wave issues NLP copies
    auto fill = [&](int st, int t) {
      const int raw = entry(t);
      const long long r0 = rows0 + (long long)(SUB ? raw & 0xffff : raw) * kTile;
      unsigned char* sp = smem + st * STAGE;
      TL::async_load(q, r0, sp, wave, goff);
      TL::async_load(dof, r0, sp + TL::BYTES, wave, goff);
      // the (lse2, Delta) operand slots of the 64 rows, 1 KiB: a quarter per wave
      lds_dma4(uniform_ptr(ldb + r0), (unsigned)(wave * 256 + lane * 4),
               __builtin_amdgcn_readfirstlane(lds0 + st * STAGE + 2 * TL::BYTES + wave * 256));
    };
    // Per-row terms folded into the matrix products: one extra MFMA step on S adds
    // -lse2[q]/sl2 (so that P = exp2(S' * sl2)) and a large negative bias on pad keys; one extra
    // step on dP subtracts Delta[q].  The preprocess kernel has split both fp32 row values into
    // three bf16 parts (exact to fp32 precision) for contraction slots 0..2; slot 3 is 1 for the S
    // step (it multiplies the key bias) and 0 for the dP step.  Only the lane half h = 0 of the
    // other operand is non-zero, so both lane halves may load the same row slots.
    bf16x8 bias_b = {0, 0, 0, 0, 0, 0, 0, 0};
    if (h == 0) {
      bias_b[0] = bias_b[1] = bias_b[2] = (__bf16)1.f;
      bias_b[3] = kvalid ? (__bf16)0.f : (__bf16)-30000.f;
    }
    // SUB: slot 3 per tile -- this lane's key row takes part iff it is valid and its key cube
    // (2*kh + (row/2)%2 of the block's four) is among those the query block of the tile selected
    const int my_sub = 2 * kh + ((l32 >> 1) & 1);
    auto set_bias = [&](int raw_entry) {
      if (!SUB) return;
      const bool on = kvalid && (((raw_entry >> 16) >> my_sub) & 1);
      uint4 u = __builtin_bit_cast(uint4, bias_b);
      u.y = h == 0 ? (0x3f80u | (on ? 0u : 0xc6ea0000u)) : 0u;  // (1, bias): bf16 1.0 and bf16(-29952)
      bias_b = __builtin_bit_cast(bf16x8, u);
    };
    auto row_read = [&](const unsigned char* stage) {
      return *(const uint4*)(stage + 2 * TL::BYTES + (qh * 32 + l32) * 16);
    };
    auto row_slots = [&](const uint4& r, bf16x8& la, bf16x8& da) {
      la = __builtin_bit_cast(bf16x8, make_uint4(r.x, r.y, 0u, 0u));
      da = __builtin_bit_cast(bf16x8, make_uint4(r.z, r.w, 0u, 0u));
    };
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // S' and dP' of the tile in stage st (prologue only; the loop interleaves the same steps)
    auto s_dp = [&](int st, f32x16& sacc, f32x16& dpacc) {
      const unsigned char* Qs = smem + st * STAGE;
      const unsigned char* Ds = Qs + TL::BYTES;
      bf16x8 la, da;
      row_slots(row_read(Qs), la, da);
      sacc = zero;
      dpacc = zero;
#pragma unroll
      for (int s = 0; s < KS; ++s) sacc = mfma32(TL::rowmajor_operand(Qs, qh * 32, s, lane), kreg[s], sacc);
      sacc = mfma32(la, bias_b, sacc);
#pragma unroll
      for (int s = 0; s < KS; ++s) dpacc = mfma32(TL::rowmajor_operand(Ds, qh * 32, s, lane), vreg[s], dpacc);
      dpacc = mfma32(da, bias_b, dpacc);
    };

    // State carried from one iteration to the next (t = tile whose dV/dK products come next):
    //   sA, dpA        S' and dP' of tile t+1
    //   pb*, sb*       P and dS of tile t as bf16 operands
    //   dt, qt         transposed dOf and Q operands of tile t
    f32x16 sA, dpA;
    // P, dS operands alternate between two register sets by iteration parity (no copies to rotate them)
    uint4 pbs[2][2], sbs[2][2];
    bf16x8 dt[DVB][2], qt[DVB][2];

    fill(0, beg);
    fill(1, beg + 1);
    fill(2, beg + 2);
    fill(3, beg + 3);
    // SUB: the entries of tiles t+2 and t+3 at the top of iteration t (iteration t forms S' of tile t+2),
    // kept from the fills that fetched them; the first two tiles are formed right here
    int ent_first = 0, ent_second = 0, ent_hist0 = 0, ent_hist1 = 0;
    if (SUB) {
      ent_first = entry(beg);
      ent_second = entry(beg + 1);
      ent_hist0 = entry(beg + 2);
      ent_hist1 = entry(beg + 3);
    }
    wait_vmcnt<2 * NLP>();
    __builtin_amdgcn_s_barrier();
    {
      f32x16 s0, dp0;
      set_bias(ent_first);
      s_dp(0, s0, dp0);
      float p[16], ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        p[i] = fast_exp2(s0[i] * sl2);
        ds[i] = p[i] * dp0[i];
      }
      pbs[0][0] = pack8(p), pbs[0][1] = pack8(p + 8);
      sbs[0][0] = pack8(ds), sbs[0][1] = pack8(ds + 8);
#pragma unroll
      for (int x = 0; x < DVB; ++x) {
        dt[x][0] = TL::transposed_operand(smem + TL::BYTES, qh * 32, 0, x * 32, lane);
        dt[x][1] = TL::transposed_operand(smem + TL::BYTES, qh * 32, 1, x * 32, lane);
        qt[x][0] = TL::transposed_operand(smem, qh * 32, 0, x * 32, lane);
        qt[x][1] = TL::transposed_operand(smem, qh * 32, 1, x * 32, lane);
      }
      set_bias(ent_second);
      s_dp(1, sA, dpA);
    }

    // One iteration, ST = stage of tile t.  Tile t+1 sits in ST+1, tile t+2 in ST+2, tile t+3 is
    // in flight and tile t+4 goes where tile t was.  Two phases, each a fixed interleave of one
    // matrix instruction with a few LDS reads, copy instructions and vector operations, so that
    // the single wavefront of a SIMD keeps the matrix pipe fed while it issues everything else:
    //   A: dV, dK of tile t          | row-major reads of tile t+2, the copies of tile t+4,
    //                                | P, dS of tile t+1
    //   B: S', dP' of tile t+2       | transposed reads of tile t+1
    const int lane_a = TL::rowmajor_lane(qh * 32, lane);
    int lane_b0, lane_b1;
    TL::transposed_lane(qh * 32, lane, lane_b0, lane_b1);
    constexpr int NA = 4 * DVB, NB = 2 * (KS + 1);
    static_assert(NA == 2 * KS && NLP <= NA && 16 % NA == 0, "phase interleave");
    auto body = [&](auto st_tag, int t) {
      constexpr int ST = decltype(st_tag)::value;
      constexpr int S1 = (ST + 1) & 3, S2 = (ST + 2) & 3;
      wait_lgkmcnt0();   // this wave's reads of tile t have landed: its stage may be overwritten
      wait_vmcnt<NLP>();  // this wave's share of tile t+2 has landed
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      const int raw4 = entry(t + 4);
      const int raw2 = ent_hist0;  // SUB: the entry of tile t+2, whose S' this iteration forms
      ent_hist0 = ent_hist1;
      ent_hist1 = raw4;
      const long long r0 = rows0 + (long long)(SUB ? raw4 & 0xffff : raw4) * kTile;
      const void* gq = uniform_ptr(q + r0 * CPR);
      const void* gd = uniform_ptr(dof + r0 * CPR);
      const void* gl = uniform_ptr(ldb + r0);
      const unsigned lq = __builtin_amdgcn_readfirstlane(lds0 + ST * STAGE + (unsigned)(wave * TL::IPW) * 1024u);
      const unsigned ll = __builtin_amdgcn_readfirstlane(lds0 + ST * STAGE + 2 * TL::BYTES + wave * 256);
      // operand addresses are rebuilt from three lane-dependent values in every iteration (one
      // XOR per read) instead of being held in registers across the loop
      int la_n = lane_a, lb0_n = lane_b0, lb1_n = lane_b1;
      asm volatile("" : "+v"(la_n), "+v"(lb0_n), "+v"(lb1_n));
      constexpr int FAR = 2 * STAGE;  // constant offsets of LDS reads stop at 64 KiB
      const int la_2 = la_n + (S2 >= 2 ? FAR : 0), lb0_1 = lb0_n + (S1 >= 2 ? FAR : 0), lb1_1 = lb1_n + (S1 >= 2 ? FAR : 0);
      const unsigned char* Q1 = smem + (S1 & 1) * STAGE;
      const unsigned char* D1 = Q1 + TL::BYTES;
      const unsigned char* Q2 = smem + (S2 & 1) * STAGE;
      const unsigned char* D2 = Q2 + TL::BYTES;
      bf16x8 qa[KS], da[KS], la, dla;
      float pn[16], dsn[16];
      uint4 rowv;
      constexpr int PAR = ST & 1;  // this iteration consumes set PAR and fills set PAR ^ 1
      auto value = [&](int i) {
        pn[i] = fast_exp2(sA[i] * sl2);
        dsn[i] = pn[i] * dpA[i];
      };
      // values [lo, hi) of P, dS; each finished pair is packed at once (few fp32 values stay live)
      auto value_step = [&](int lo, int hi) {
#pragma unroll
        for (int e = lo; e < hi; ++e) {
          value(e);
          if (e & 1) {
            const uint32_t pp = pack_bf16(pn[e - 1], pn[e]), ss = pack_bf16(dsn[e - 1], dsn[e]);
            uint4& pu = pbs[PAR ^ 1][e >> 3];
            uint4& su = sbs[PAR ^ 1][e >> 3];
            const int w = (e >> 1) & 3;
            if (w == 0) pu.x = pp, su.x = ss;
            if (w == 1) pu.y = pp, su.y = ss;
            if (w == 2) pu.z = pp, su.z = ss;
            if (w == 3) pu.w = pp, su.w = ss;
            // pure arithmetic has no place of its own in the instruction order: tie it to this step
            asm volatile("" : : "v"(pp), "v"(ss));
          }
        }
      };

#pragma unroll
      for (int i = 0; i < NA; ++i) {
        const int x = i >> 2, sub = i & 3;
        if (sub == 0) dva[x] = mfma32(dt[x][0], __builtin_bit_cast(bf16x8, pbs[PAR][0]), dva[x]);
        if (sub == 1) dva[x] = mfma32(dt[x][1], __builtin_bit_cast(bf16x8, pbs[PAR][1]), dva[x]);
        if (sub == 2) dka[x] = mfma32(qt[x][0], __builtin_bit_cast(bf16x8, sbs[PAR][0]), dka[x]);
        if (sub == 3) dka[x] = mfma32(qt[x][1], __builtin_bit_cast(bf16x8, sbs[PAR][1]), dka[x]);
        if (i < KS) qa[i] = TL::rowmajor_at(Q2, la_2, i);
        else da[i - KS] = TL::rowmajor_at(D2, la_2, i - KS);
        if (i == 0) rowv = row_read(smem + S2 * STAGE);
        // copies of tile t+4: one M0 value per tensor, the 1 KiB steps ride in the instruction offset
        if (i == 0) set_m0(lq);
        if (i == TL::IPW) set_m0(lq + TL::BYTES);
        if (i < 2 * TL::IPW) {
          const void* g = i < TL::IPW ? gq : gd;
          const int r = i % TL::IPW;
          if (r == 0) lds_dma16_at<0>(g, goff[0]);
          if (r == 1) lds_dma16_at<1024>(g, goff[1 % TL::IPW]);
          if (r == 2) lds_dma16_at<2048>(g, goff[2 % TL::IPW]);
          if (r == 3) lds_dma16_at<3072>(g, goff[3 % TL::IPW]);
        } else if (i == 2 * TL::IPW) lds_dma4(gl, (unsigned)(wave * 256 + lane * 4), ll);
        value_step(i * 16 / NA, (i + 1) * 16 / NA);  // P, dS of tile t+1 (S', dP' of it die here)
        __builtin_amdgcn_sched_barrier(0);
      }
      f32x16 sN, dpN;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int s = i >> 1;
        if (!(i & 1)) sN = mfma32(s < KS ? qa[s < KS ? s : 0] : la, s < KS ? kreg[s < KS ? s : 0] : bias_b, i < 2 ? zero : sN);
        else dpN = mfma32(s < KS ? da[s < KS ? s : 0] : dla, s < KS ? vreg[s < KS ? s : 0] : bias_b, i < 2 ? zero : dpN);
        if (i < 4 * DVB) {
          const int x = i >> 2, which = i & 3;
          if (which < 2) dt[x][which] = TL::transposed_at(D1, lb0_1, lb1_1, which, x);
          else qt[x][which - 2] = TL::transposed_at(Q1, lb0_1, lb1_1, which - 2, x);
        }
        if (i == NB - 4) {  // the operands of the two bias steps are put together here, not earlier
          asm volatile("" : "+v"(rowv.x), "+v"(rowv.y), "+v"(rowv.z), "+v"(rowv.w));
          row_slots(rowv, la, dla);
          set_bias(raw2);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      sA = sN;
      dpA = dpN;
    };

    for (int t = beg; t < end; t += 4) {
      body(std::integral_constant<int, 0>{}, t);
      if (t + 1 < end) body(std::integral_constant<int, 1>{}, t + 1);
      if (t + 2 < end) body(std::integral_constant<int, 2>{}, t + 2);
      if (t + 3 < end) body(std::integral_constant<int, 3>{}, t + 3);
    }
    wait_vmcnt<0>();  // the refetches issued past the end of the list
  }
  // the pooled-gradient terms of this thread's column chunk (the same chunk for all of its items),
  // requested before the partial results go through LDS
  static_assert(256 % CPR == 0, "a thread keeps its column chunk");
  float4 pk[2] = {}, pv[2] = {};
  if (!SUB) {
    const float* a = dkc + ((bh * Nc + j) / m_blocks) * D + (tid % CPR) * 8;  // per cube = m_blocks blocks
    const float* b = dvc + ((bh * Nc + j) / m_blocks) * D + (tid % CPR) * 8;
    pk[0] = *(const float4*)a, pk[1] = *(const float4*)(a + 4);
    pv[0] = *(const float4*)b, pv[1] = *(const float4*)(b + 4);
  }
  __syncthreads();

  // merge the two query halves: all four partial results (dK, dV x two query halves) go through LDS at once
  const float inv_cnt = 1.0f / (float)cube_count(mask, j, m_blocks);
  static_assert(4 * 64 * OS * 4 <= 4 * STAGE, "merge buffers must fit");
  float* parts_lds = (float*)smem;  // [dK half 0][dK half 1][dV half 0][dV half 1], each [64][OS]
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    float* Op = parts_lds + (pass * 2 + qh) * 64 * OS + kh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const f32x16& a = pass == 0 ? dka[x] : dva[x];
        float4 val = make_float4(a[4 * g4], a[4 * g4 + 1], a[4 * g4 + 2], a[4 * g4 + 3]);
        *(float4*)&Op[merge_offset(l32, x * 32 + 8 * g4 + 4 * h, OS)] = val;
      }
  }
  __syncthreads();
  if (slot >= 0) {  // one run of a split list: raw fp32 sums [dK | dV][64][D], finished by k_dkv_reduce
    float* dst = parts + ((bh * cap + slot) * 2) * (long long)(64 * D);
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const float* part0 = parts_lds + pass * 2 * 64 * OS;
      const float* part1 = part0 + 64 * OS;
#pragma unroll
      for (int it = 0; it < LPT; ++it) {
        const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
        const int m0 = merge_offset(r, ch * 8, OS), m1 = merge_offset(r, ch * 8 + 4, OS);
        const float4 a0 = *(const float4*)(part0 + m0), a1 = *(const float4*)(part0 + m1);
        const float4 b0 = *(const float4*)(part1 + m0), b1 = *(const float4*)(part1 + m1);
        float4* o = (float4*)(dst + pass * 64 * D + r * D + ch * 8);
        o[0] = make_float4(a0.x + b0.x, a0.y + b0.y, a0.z + b0.z, a0.w + b0.w);
        o[1] = make_float4(a1.x + b1.x, a1.y + b1.y, a1.z + b1.z, a1.w + b1.w);
      }
    }
    return;
  }
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const float4 p0 = pass == 0 ? pk[0] : pv[0], p1 = pass == 0 ? pk[1] : pv[1];
    const float pooled[8] = {p0.x * inv_cnt, p0.y * inv_cnt, p0.z * inv_cnt, p0.w * inv_cnt,
                             p1.x * inv_cnt, p1.y * inv_cnt, p1.z * inv_cnt, p1.w * inv_cnt};
    const float mul = pass == 0 ? scale : 1.0f;
    uint4* dst = pass == 0 ? dk : dv;
    const float* part0 = parts_lds + pass * 2 * 64 * OS;
    const float* part1 = part0 + 64 * OS;
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
      const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
      const int m0 = merge_offset(r, ch * 8, OS), m1 = merge_offset(r, ch * 8 + 4, OS);
      const float4 a0 = *(const float4*)(part0 + m0), a1 = *(const float4*)(part0 + m1);
      const float4 b0 = *(const float4*)(part1 + m0), b1 = *(const float4*)(part1 + m1);
      const float sum[8] = {a0.x + b0.x, a0.y + b0.y, a0.z + b0.z, a0.w + b0.w, a1.x + b1.x, a1.y + b1.y, a1.z + b1.z, a1.w + b1.w};
      uint4 ov = make_uint4(0, 0, 0, 0);
      if ((kmask >> r) & 1) {
        float res[8];
        if (SUB) {
          float pl[8];
          subcube_pooled_term(pass == 0 ? dkc : dvc, (bh * Nc + j) * 4, kmask, r, D, ch, pl);
#pragma unroll
          for (int e = 0; e < 8; ++e) res[e] = fmaf(sum[e], mul, pl[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) res[e] = fmaf(sum[e], mul, pooled[e]);
        }
        ov = pack8(res);
      }
      dst[(rows0 + j * kTile + r) * CPR + ch] = ov;
    }
  }
}

// Sums the fp32 partial results of the split lists in slot order and finishes them like the dK/dV
// epilogue does (scale, pooled-gradient term, zero pad rows, one rounding to bf16).  One workgroup
// per possible split list of a (b, h); those beyond the actual number exit at once.
template <int D, bool SUB>
__global__ __launch_bounds__(256) void k_dkv_reduce(int Nc, int cap, float scale, const int32_t* __restrict__ split,
                                                    const float* __restrict__ parts, const float* __restrict__ dkc,
                                                    const float* __restrict__ dvc, const uint64_t* __restrict__ mask,
                                                    uint4* __restrict__ dk, uint4* __restrict__ dv, int m_blocks) {
  constexpr int CPR = D / 8, LPT = kTile * CPR / 256;
  const int per = cap / 2, r_ = blockIdx.x % per, tid = threadIdx.x;
  const long long bh = blockIdx.x / per;
  const int4* sp = (const int4*)split + bh * (per + 1);
  if (r_ >= sp[0].x) return;
  const int4 desc = sp[1 + r_];
  const int j = desc.x, slot0 = desc.y, runs = desc.z;
  const uint64_t kmask = mask[j];
  const float inv_cnt = 1.0f / (float)cube_count(mask, j, m_blocks);
  const long long rows0 = bh * (long long)Nc * kTile;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const float* pooled_row = (pass == 0 ? dkc : dvc) + ((bh * Nc + j) / m_blocks) * D + (tid % CPR) * 8;
    const float4 p0 = *(const float4*)pooled_row, p1 = *(const float4*)(pooled_row + 4);
    const float pooled[8] = {p0.x * inv_cnt, p0.y * inv_cnt, p0.z * inv_cnt, p0.w * inv_cnt,
                             p1.x * inv_cnt, p1.y * inv_cnt, p1.z * inv_cnt, p1.w * inv_cnt};
    const float mul = pass == 0 ? scale : 1.0f;
    uint4* dst = pass == 0 ? dk : dv;
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
      const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
      float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int s = 0; s < runs; ++s) {
        const float4* src = (const float4*)(parts + (((bh * cap + slot0 + s) * 2 + pass) * 64 + r) * (long long)D + ch * 8);
        const float4 a = src[0], b = src[1];
        sum[0] += a.x; sum[1] += a.y; sum[2] += a.z; sum[3] += a.w;
        sum[4] += b.x; sum[5] += b.y; sum[6] += b.z; sum[7] += b.w;
      }
      uint4 ov = make_uint4(0, 0, 0, 0);
      if ((kmask >> r) & 1) {
        float res[8];
        if (SUB) {
          float pl[8];
          subcube_pooled_term(pass == 0 ? dkc : dvc, (bh * Nc + j) * 4, kmask, r, D, ch, pl);
#pragma unroll
          for (int e = 0; e < 8; ++e) res[e] = fmaf(sum[e], mul, pl[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) res[e] = fmaf(sum[e], mul, pooled[e]);
        }
        ov = pack8(res);
      }
      dst[(rows0 + j * kTile + r) * CPR + ch] = ov;
    }
  }
}

hipError_t launch_fine_bwd_dkv(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                               const void* dof, const int32_t* col, const int32_t* order, const int32_t* split,
                               float* parts, int cap, const void* ldb, const float* dkc, const float* dvc,
                               const uint64_t* mask, void* dk, void* dv, int m_blocks, int key_cubes_16, hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const int items = Nc + cap;
  const unsigned grid = (unsigned)(BH * items), rgrid = (unsigned)(BH * (cap / 2));
#define VSA_DKV(D_, SUB_)                                                                                                \
  do {                                                                                                                   \
    k_fine_bwd_dkv<D_, SUB_><<<grid, 256, 0, s>>>(Nc, K, sl2, scale, (const uint4*)q, (const uint4*)k, (const uint4*)v,    \
                                                  (const uint4*)dof, col, order, items, parts, cap, (const uint4*)ldb,   \
                                                  dkc, dvc, mask, (uint4*)dk, (uint4*)dv, m_blocks);                      \
    k_dkv_reduce<D_, SUB_><<<rgrid, 256, 0, s>>>(Nc, cap, scale, split, parts, dkc, dvc, mask, (uint4*)dk, (uint4*)dv,    \
                                                 m_blocks);                                                              \
  } while (0)
  if (key_cubes_16) {  // lists of key cubes of 16 tokens: the pooled terms dkc, dvc are [BH, 4 Nc, d]
    if (d == 128) VSA_DKV(128, true);
    else VSA_DKV(64, true);
  } else {
    if (d == 128) VSA_DKV(128, false);
    else VSA_DKV(64, false);
  }
#undef VSA_DKV
  return hipGetLastError();
}

}  // namespace vsa
