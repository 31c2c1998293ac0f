// Fine stage forward (Sec. 2.2 fine stage; Sec. 2.1 attention equation under the block mask)
// fused with the gated combine O = O_c * G_c + O_f * G_f.
//
// One workgroup (4 wavefronts) per (b, h, 64-row query block); "cube" below means such a block (a
// cube of 64*m tokens is m consecutive blocks, and the lists the kernel gets name blocks).  The K
// selected key blocks are walked through a double-buffered LDS stage (K tile + V tile).  LIST says how
// list entries turn into streamed 64-key tiles: CubeList, one entry = one block; SubCubeList, four
// entries that name key cubes of 16 tokens are gathered into one tile (Sec. 3.2, 64 x 16 tiles).  Work split inside the workgroup:
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
#include <type_traits>

#include "fine_tile.h"
#include "vsa_kernels.h"

namespace vsa {

constexpr float kMaskBias = -30000.f;  // added to the raw logits of pad keys (|q.k| is assumed < 15000)
constexpr float kTau = 8.f;             // lazy-rescale threshold, log2 units

// max over both lane halves (lanes l and l^32) with one cross-lane VALU instruction instead of a
// round trip through the LDS permute path
__device__ __forceinline__ float max_across_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int D, class LIST>
__global__ __launch_bounds__(256, 2) void k_fine_fwd(int Nc, int K, float sl2, const uint4* __restrict__ q,
                                                     const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                     const uint4* __restrict__ gc, const uint4* __restrict__ gf,
                                                     const int32_t* __restrict__ idx, const float* __restrict__ oc,
                                                     const uint64_t* __restrict__ mask, uint4* __restrict__ out,
                                                     uint4* __restrict__ out_fine, float* __restrict__ lse_f,
                                                     int H, long long out_head_stride, long long out_row_stride,
                                                     int m_blocks) {
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

  // With K = Nc every workgroup of a head walks the same list: then all XCDs work on the same head
  // (plain blockIdx order), which keeps that list's tiles shared chip-wide, and the workgroups that
  // run side by side on an XCD (cubes c, c+8, ...) start their walk a few entries apart and wrap
  // around -- otherwise they ask for the same cache lines in the same cycles.
  // (The walk is in tiles of 64 keys: one list entry, or four entries that name key cubes of 16 tokens.)
  const int NT = (K + LIST::kEntriesPerTile - 1) / LIST::kEntriesPerTile;
  const bool same_lists = K == Nc * LIST::kEntriesPerTile;
  const unsigned wg = same_lists ? blockIdx.x : xcd_chunked_id(blockIdx.x, gridDim.x);
  const int c = wg % Nc;
  const long long bh = wg / Nc;
  const int rot = same_lists ? ((c >> 3) & 15) % NT : 0;
  auto ent = [&](int t) { const int e = t + rot; return e >= NT ? e - NT : e; };
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qh = wave & 1, kh = wave >> 1, l32 = lane & 31, h = lane >> 5;
  const long long rows0 = bh * (long long)Nc * kTile;  // first row of this (b,h)
  const int32_t* my_idx = idx + (bh * Nc + c) * (long long)K;

  // Software pipeline of the K/V stream: two LDS stages (K tile + V tile each), the copy of tile
  // t+1 runs behind the math of tile t.  Per tile: wait for this wave's share of tile t, one
  // barrier (tile t complete; every wave is done with tile t-1), start the copy of tile t+1 into
  // the other stage, do the math with operands read from LDS just ahead of their use.
  // The barrier is a raw s_barrier (no fence): a fence would drain the copy still in flight.
  // vmcnt is waited by hand (the compiler cannot see the copies; see Tile::async_load).
  unsigned goff[TL::IPW];
  LIST::template offsets<TL>(wave, lane, goff);
  auto issue = [&](unsigned char* st, int row) {  // `row`: first source row of this wave's share
    TL::async_load(k, rows0 + row, st, wave, goff);
    TL::async_load(v, rows0 + row, st + TL::BYTES, wave, goff);
  };
  // Start-up order: the list first (one round trip), then the copy of tile 0, and only then the
  // loads of the key masks and of Q, so that everything the first iteration needs is in flight
  // together.  The empty asm below consumes the loaded registers: the compiler has to place its
  // wait for them right there (it also drains the copy), and its own vmcnt bookkeeping has nothing
  // left to wait for inside the loop.
  LIST cubes;
  cubes.init(my_idx, mask, K, kh, wave, lane, Nc);
  issue(stage0, cubes.first_row(ent(0)));
  cubes.load_masks();
  bf16x8 qreg[KS];
  {
    const uint4* qrow = q + (rows0 + c * kTile + qh * 32 + l32) * CPR;
#pragma unroll
    for (int s = 0; s < KS; ++s) qreg[s] = __builtin_bit_cast(bf16x8, qrow[2 * s + h]);
  }
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(qreg[s]));
  asm volatile("" : "+v"(cubes.km_v));
  uint32_t km_cur;  // valid-key mask (this wave's key half) of the tile of this iteration
  {
    int j0;
    cubes.get_tile(ent(0), j0, km_cur);
  }
  const int lane_a = TL::rowmajor_lane(kh * 32, lane);
  int lane_b0, lane_b1;
  TL::transposed_lane(kh * 32, lane, lane_b0, lane_b1);

  float mref = -INFINITY, lsum = 0.f;
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16x8 ones_b = zero8;
  ones_b[0] = (h == 0) ? (__bf16)1.f : (__bf16)0.f;
  f32x16 o[DVB];
#pragma unroll
  for (int x = 0; x < DVB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[x][i] = 0.f;

  auto body = [&](auto copy_tag, const unsigned char* cur, unsigned char* nxt, int t) {
    constexpr bool COPY = decltype(copy_tag)::value;  // false for the last tile of the list
    const uint32_t kmask = km_cur;
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    // The copy of the next tile is not issued in one burst here -- eight wavefronts doing that at
    // the same moment queue up behind one another in the load path and stall -- but one
    // instruction per S^T step below.
    int jn = 0;
    if (COPY) cubes.get_tile(ent(t + 1), jn, km_cur);
    const void* gk = uniform_ptr(k + (rows0 + jn) * CPR);
    const void* gv = uniform_ptr(v + (rows0 + jn) * CPR);
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
    constexpr int PIECES_PER_STEP = (2 * TL::IPW + KS - 1) / KS;
    __builtin_amdgcn_sched_barrier(0);
    const unsigned char* Ks = cur;
    const unsigned char* Vs = cur + TL::BYTES;
    // Operand i: K rows (S^T steps), then transposed V (O^T steps).  The K operands are requested a
    // fixed number of matrix instructions ahead of their use, the V operands during the last S^T
    // steps and the softmax arithmetic; addresses are rebuilt from three lane values (one XOR each).
    int la = lane_a, lb0 = lane_b0, lb1 = lane_b1;
    asm volatile("" : "+v"(la), "+v"(lb0), "+v"(lb1));
    constexpr int NOP = KS + 2 * DVB, AHEAD = 4;
    bf16x8 op[NOP];
    auto read_op = [&](int i) {
      if (i < KS) return TL::rowmajor_at(Ks, la, i);
      const int j = i - KS;
      return TL::transposed_at(Vs, lb0, lb1, j & 1, j >> 1);
    };
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) op[i] = read_op(i);
    __builtin_amdgcn_sched_barrier(0);

    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      sacc = mfma32(op[i], qreg[i], sacc);
      op[i + AHEAD] = read_op(i + AHEAD);
#pragma unroll
      for (int c2 = 0; c2 < PIECES_PER_STEP; ++c2) copy_piece(i * PIECES_PER_STEP + c2);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = KS + AHEAD; i < NOP; ++i) op[i] = read_op(i);

    // Pad keys of a partially filled cube never take part: one extra MFMA adds a large negative
    // bias to their rows of S^T (A = bias of key l%32 in contraction slot 0, B = ones in slot 0).
    const bool partial = kmask != 0xffffffffu;
    if (partial) {
      const bool dead = !((kmask >> l32) & 1);
      bf16x8 ab = zero8;
      ab[0] = (h == 0 && dead) ? (__bf16)kMaskBias : (__bf16)0.f;
      sacc = mfma32(ab, ones_b, sacc);
    }

    // Online softmax with a lazily updated reference maximum: mref only moves when the running
    // maximum exceeds it by more than kTau (log2 units), so exp2(s - mref) stays below 2^kTau and
    // the O / l rescale is skipped for almost every tile.  The result is exact either way.
    float mx = fmaxf(fmaxf(sacc[0], sacc[1]), sacc[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, sacc[i]), sacc[i + 1]);
    mx = fmaxf(mx, sacc[15]);
    mx = max_across_halves(mx);
    if (partial && mx < 0.5f * kMaskBias) mx = -INFINITY;  // every key of this half is a pad
    const float mx2 = mx * sl2;
    if (__any(mx2 > mref + kTau)) {
      // only the lanes over the threshold move their reference: a lane's arithmetic then never
      // depends on what other query columns (pad rows included) hold
      const float mnew = (mx2 > mref + kTau) ? mx2 : mref;
      // mref = -inf: nothing accumulated yet, the factor is irrelevant but must not be NaN
      const float alpha = (mnew == -INFINITY) ? 1.f : fast_exp2(mref - mnew);
      lsum *= alpha;
#pragma unroll
      for (int x = 0; x < DVB; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[x][i] *= alpha;
      mref = mnew;
    }
    const float muse = (mref == -INFINITY) ? 0.f : mref;
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = fast_exp2(fmaf(sacc[i], sl2, -muse));
      lsum += p[i];
    }
    const bf16x8 pb0 = acc_to_operand(p), pb1 = acc_to_operand(p + 8);
#pragma unroll
    for (int x = 0; x < DVB; ++x) {
      o[x] = mfma32(op[KS + 2 * x], pb0, o[x]);
      o[x] = mfma32(op[KS + 2 * x + 1], pb1, o[x]);
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
  __syncthreads();

  // `out` may be head-major [B,H,Np,D] or token-major [B,Np,H,D] (same batch stride): chunk ch of
  // tiled row n of head h of batch b sits at b*H*Np*CPR + h*out_head_stride + n*out_row_stride + ch
  const long long out0 = (bh / H) * ((long long)H * Nc * kTile * CPR) + (bh % H) * out_head_stride;
  // ---- merge the two key halves, normalise, gate, store
  // The gates and the coarse output of this thread's items are requested first: they arrive while
  // the partial results go through LDS.  Pad rows are loaded too (they exist in memory) and ignored.
  const uint64_t qmask = mask[c];
  uint4 gc_raw[LPT], gf_raw[LPT];
  float4 oc_raw[LPT][2];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
    const long long g = (rows0 + c * kTile + r) * CPR + ch;
    const float* ocr = oc + ((bh * Nc + c) / m_blocks) * D + ch * 8;  // O_c is per cube = m_blocks blocks
    gc_raw[it] = gc[g];
    gf_raw[it] = gf ? gf[g] : make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);  // bf16 ones
    oc_raw[it][0] = *(const float4*)ocr;
    oc_raw[it][1] = *(const float4*)(ocr + 4);
  }
  // Partial O of wave (qh, kh) goes to rows qh*32.. of stage `kh` (fp32 [64][D] each).
  lsum += __shfl_xor(lsum, 32);
  {
    float* Op = (float*)(kh == 0 ? stage0 : stage1) + qh * 32 * OS;
#pragma unroll
    for (int x = 0; x < DVB; ++x)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float4 val = make_float4(o[x][4 * g4], o[x][4 * g4 + 1], o[x][4 * g4 + 2], o[x][4 * g4 + 3]);
        *(float4*)&Op[merge_offset(l32, x * 32 + 8 * g4 + 4 * h, OS)] = val;
      }
  }
  if (h == 0) {
    ml[(wave * 32 + l32) * 2] = mref;
    ml[(wave * 32 + l32) * 2 + 1] = lsum;
  }
  __syncthreads();

#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int item = it * 256 + tid, r = item / CPR, ch = item % CPR;
    const int wa = r >> 5, wb = wa + 2, ql = r & 31;
    const float ma = ml[(wa * 32 + ql) * 2], la = ml[(wa * 32 + ql) * 2 + 1];
    const float mb = ml[(wb * 32 + ql) * 2], lb = ml[(wb * 32 + ql) * 2 + 1];
    const float M = fmaxf(ma, mb);
    // (M = -inf: the list named no valid key at all -- only a caller-supplied list can, e.g. one made of
    // dead key cubes; the row then gets O_f = 0 and lse = 0 instead of NaN)
    const bool none = M == -INFINITY;
    float fa = none ? 0.f : fast_exp2(ma - M), fb = none ? 0.f : fast_exp2(mb - M);
    const float inv = none ? 0.f : 1.0f / (la * fa + lb * fb);
    fa *= inv; fb *= inv;
    const int m0 = merge_offset(r, ch * 8, OS), m1 = merge_offset(r, ch * 8 + 4, OS);
    const float* Oa = (const float*)stage0;
    const float* Ob = (const float*)stage1;
    float of[8], res[8];
    const float4 a0 = *(const float4*)(Oa + m0), a1 = *(const float4*)(Oa + m1);
    const float4 b0 = *(const float4*)(Ob + m0), b1 = *(const float4*)(Ob + m1);
    of[0] = a0.x * fa + b0.x * fb; of[1] = a0.y * fa + b0.y * fb; of[2] = a0.z * fa + b0.z * fb; of[3] = a0.w * fa + b0.w * fb;
    of[4] = a1.x * fa + b1.x * fb; of[5] = a1.y * fa + b1.y * fb; of[6] = a1.z * fa + b1.z * fb; of[7] = a1.w * fa + b1.w * fb;
    const long long g = (rows0 + c * kTile + r) * CPR + ch;
    const bool valid = (qmask >> r) & 1;
    uint4 ov = make_uint4(0, 0, 0, 0), fv = make_uint4(0, 0, 0, 0);
    if (valid) {
      float gcv[8], gfv[8];
      unpack8(gc_raw[it], gcv);
      unpack8(gf_raw[it], gfv);
      const float4 c0 = oc_raw[it][0], c1 = oc_raw[it][1];
      const float ocv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) res[e] = fmaf(ocv[e], gcv[e], of[e] * gfv[e]);
      ov = pack8(res);
      fv = pack8(of);
    }
    out[out0 + (long long)(c * kTile + r) * out_row_stride + ch] = ov;
    if (out_fine) out_fine[g] = fv;
  }
  if (lse_f && tid < kTile) {
    const int r = tid, wa = r >> 5, wb = wa + 2, ql = r & 31;
    const float ma = ml[(wa * 32 + ql) * 2], la = ml[(wa * 32 + ql) * 2 + 1];
    const float mb = ml[(wb * 32 + ql) * 2], lb = ml[(wb * 32 + ql) * 2 + 1];
    const float M = fmaxf(ma, mb);
    const float Lt = la * fast_exp2(ma - M) + lb * fast_exp2(mb - M);
    lse_f[rows0 + c * kTile + r] = (((qmask >> r) & 1) && M != -INFINITY) ? (M + fast_log2(Lt)) * kLn2 : 0.f;
  }
}

hipError_t launch_fine_fwd(int BH, int Nc, int d, int K, float scale, const void* q, const void* k, const void* v,
                           const void* gate_c, const void* gate_f, const int32_t* idx, const float* oc,
                           const uint64_t* mask, void* out, void* out_fine, float* lse_f, int H, int out_token_major,
                           int m_blocks, int key_cubes_16, hipStream_t s) {
  const float sl2 = scale * kLog2e;
  const unsigned grid = (unsigned)(BH * Nc);
  const long long cpr = d / 8, Np = (long long)Nc * kTile;
  const long long ohs = out_token_major ? cpr : Np * cpr, ors = out_token_major ? H * cpr : cpr;
#define VSA_FWD(D_, LIST_)                                                                                           \
  k_fine_fwd<D_, LIST_><<<grid, 256, 0, s>>>(Nc, K, sl2, (const uint4*)q, (const uint4*)k, (const uint4*)v,           \
                                             (const uint4*)gate_c, (const uint4*)gate_f, idx, oc, mask, (uint4*)out, \
                                             (uint4*)out_fine, lse_f, H, ohs, ors, m_blocks)
  if (key_cubes_16) {  // K counts key cubes of 16 tokens
    if (d == 128) VSA_FWD(128, SubCubeList);
    else VSA_FWD(64, SubCubeList);
  } else {
    if (d == 128) VSA_FWD(128, CubeList);
    else VSA_FWD(64, CubeList);
  }
#undef VSA_FWD
  return hipGetLastError();
}

}  // namespace vsa
