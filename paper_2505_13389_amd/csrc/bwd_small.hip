// Small backward steps: the elementwise preprocess, the coarse-stage backward (fp32) and the
// transposed block map.  The gradient formulas are the chain rule through Sec. 2.2's gated sum,
// coarse softmax attention and mean pooling.
#include "gemm32_tile.h"
#include "list_rules.h"
#include "vsa_kernels.h"

namespace vsa {

// ---------------------------------------------------------------------------------------------
// Preprocess.  Per token i of cube c (pad rows produce zeros):
//   dGc_i = dO_i * Oc[c]      dGf_i = dO_i * Of_i      dOf_i = dO_i * Gf_i  (bf16, feeds the MFMAs)
//   Delta_i = sum_d dOf_i * Of_i                       dOc[c] = sum_i dO_i * Gc_i
//   ld_i = (lse_i * log2(e), Delta_i) as one pair per row, lse = +inf on pad rows (makes P = 0
//          there in the fine backward kernels)
// One workgroup per (b*h, cube), which walks the cube's m blocks of 64 rows; thread layout as in the
// pooling kernel.
template <int D>
__global__ __launch_bounds__(256) void k_bwd_pre(int Nc, int m_blocks, const uint64_t* __restrict__ mask, const uint4* __restrict__ dout,
                                                 const uint4* __restrict__ gc, const uint4* __restrict__ gf,
                                                 const uint4* __restrict__ of, const float* __restrict__ oc,
                                                 uint4* __restrict__ dgc, uint4* __restrict__ dgf,
                                                 uint4* __restrict__ dof, float* __restrict__ ld,
                                                 uint4* __restrict__ ldb, float inv_sl2, float* __restrict__ doc,
                                                 const float* __restrict__ lse_f, int H, long long do_head_stride,
                                                 long long do_row_stride) {
  constexpr int CPR = D / 8, RG = 256 / CPR, RPT = kTile / RG;
  __shared__ float part[RG][D + 4];
  const int c = blockIdx.x % Nc;
  const long long bh = blockIdx.x / Nc;
  const int ch = threadIdx.x % CPR, rg = threadIdx.x / CPR;
  float ocv[8];
  {
    const float* p = oc + (bh * Nc + c) * D + ch * 8;
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    ocv[0] = a.x; ocv[1] = a.y; ocv[2] = a.z; ocv[3] = a.w; ocv[4] = b.x; ocv[5] = b.y; ocv[6] = b.z; ocv[7] = b.w;
  }
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int sb = 0; sb < m_blocks; ++sb) {
  const long long blk = (bh * Nc + c) * m_blocks + sb;  // block index over all (b, h)
  const uint64_t m = mask[c * m_blocks + sb];
  const long long row0 = blk * (long long)kTile;
  // dout may be head-major [B,H,Np,D] or token-major [B,Np,H,D] (see the forward's `out`)
  const long long Npad = (long long)Nc * m_blocks * kTile;
  const long long do0 = (bh / H) * ((long long)H * Npad * CPR) + (bh % H) * do_head_stride +
                        ((long long)c * m_blocks + sb) * kTile * do_row_stride;
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg + i * RG;
    const long long g = (row0 + r) * CPR + ch;
    const bool valid = (m >> r) & 1;
    uint4 z = make_uint4(0, 0, 0, 0), o_gc = z, o_gf = z, o_dof = z;
    float dsum = 0.f;
    if (valid) {
      float go[8], gcv[8], gfv[8], ofv[8], t0[8], t1[8], t2[8];
      unpack8(dout[do0 + r * do_row_stride + ch], go);
      unpack8(gc[g], gcv);
      unpack8(of[g], ofv);
      if (gf) unpack8(gf[g], gfv);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) gfv[e] = 1.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        t0[e] = go[e] * ocv[e];
        t1[e] = go[e] * ofv[e];
        t2[e] = go[e] * gfv[e];
        acc[e] += go[e] * gcv[e];
      }
      o_gc = pack8(t0); o_gf = pack8(t1); o_dof = pack8(t2);
      float t2r[8];
      unpack8(o_dof, t2r);  // Delta uses the rounded dOf, the value the fine kernels multiply with
#pragma unroll
      for (int e = 0; e < 8; ++e) dsum = fmaf(t2r[e], ofv[e], dsum);
    }
    dgc[g] = o_gc;
    if (dgf) dgf[g] = o_gf;
    dof[g] = o_dof;
#pragma unroll
    for (int o = CPR / 2; o > 0; o >>= 1) dsum += __shfl_xor(dsum, o);
    if (ch == 0) {
      const float lse2 = valid ? lse_f[row0 + r] * kLog2e : INFINITY;
      *(float2*)&ld[2 * (row0 + r)] = make_float2(lse2, dsum);
      // the same pair as two rows of bf16 MFMA operand slots: -lse2/sl2 and -Delta, each split into
      // three bf16 parts that add up to the fp32 value, then a constant slot (1 for the first, 0
      // for the second).  Pad rows carry a large finite negative number instead of -inf.
      const uint2 a = split3_bf16(valid ? -lse2 * inv_sl2 : -30000.f, 1.f);
      const uint2 b = split3_bf16(-dsum, 0.f);
      ldb[row0 + r] = make_uint4(a.x, a.y, b.x, b.y);
    }
  }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][ch * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0;
    for (int r = 0; r < RG; ++r) s += part[r][threadIdx.x];
    doc[(bh * Nc + c) * D + threadIdx.x] = s;
  }
}

hipError_t launch_bwd_pre(int BH, int Nc, int m_blocks, int d, const uint64_t* mask, const void* dout, const void* gate_c,
                          const void* gate_f, const void* out_fine, const float* oc, void* dgate_c, void* dgate_f,
                          void* dof, float* ld, void* ldb, float scale, float* doc, const float* lse_f, int H,
                          int dout_token_major, hipStream_t s) {
  const unsigned grid = (unsigned)(BH * Nc);
  const float inv_sl2 = 1.0f / (scale * kLog2e);
  const long long cpr = d / 8, Np = (long long)Nc * m_blocks * kTile;
  const long long dhs = dout_token_major ? cpr : Np * cpr, drs = dout_token_major ? H * cpr : cpr;
  if (d == 128)
    k_bwd_pre<128><<<grid, 256, 0, s>>>(Nc, m_blocks, mask, (const uint4*)dout, (const uint4*)gate_c, (const uint4*)gate_f,
                                        (const uint4*)out_fine, oc, (uint4*)dgate_c, (uint4*)dgate_f, (uint4*)dof, ld,
                                        (uint4*)ldb, inv_sl2, doc, lse_f, H, dhs, drs);
  else
    k_bwd_pre<64><<<grid, 256, 0, s>>>(Nc, m_blocks, mask, (const uint4*)dout, (const uint4*)gate_c, (const uint4*)gate_f,
                                       (const uint4*)out_fine, oc, (uint4*)dgate_c, (uint4*)dgate_f, (uint4*)dof, ld,
                                       (uint4*)ldb, inv_sl2, doc, lse_f, H, dhs, drs);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Up to three independent problems of the same shape run as one launch (blockIdx.z = problem *
// batch + batch index): the small coarse-stage products do not fill the chip one at a time.
struct GemmOperands {
  const float* a; long long sab; int sam, sak;
  const float* b; long long sbb; int sbk, sbn;
  float* c; long long scb; float alpha;
};
struct GemmSet { GemmOperands p[3]; };

__global__ __launch_bounds__(256) void k_gemm32(int M, int N, int Kd, int batch, GemmSet set) {
  __shared__ __attribute__((aligned(16))) float As[64][36];
  __shared__ __attribute__((aligned(16))) float Bs[64][36];
  const GemmOperands& g = set.p[blockIdx.z / batch];
  const int b = blockIdx.z % batch, m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int sam = g.sam, sak = g.sak, sbk = g.sbk, sbn = g.sbn;
  const float* ab = g.a + b * g.sab + (long long)m0 * sam;
  const float* bb = g.b + b * g.sbb + (long long)n0 * sbn;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1, l32 = lane & 31, h = lane >> 5;
  f32x16g acc;
  gemm_tile_global(As, Bs, ab, sam, sak, M - m0, bb, sbn, sbk, N - n0, Kd, tid, acc);
  float* cb = g.c + b * g.scb;
  const float alpha = g.alpha;
  const int n = n0 + wn * 32 + l32;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = m0 + wm * 32 + 8 * (i / 4) + 4 * h + (i % 4);
    if (m < M && n < N) cb[(long long)m * N + n] = alpha * acc[i];
  }
}

static GemmOperands gemm_operands(float alpha, const float* a, long long sab, int sam, int sak, const float* b,
                                  long long sbb, int sbk, int sbn, float* c, long long scb) {
  GemmOperands o;
  o.a = a; o.sab = sab; o.sam = sam; o.sak = sak;
  o.b = b; o.sbb = sbb; o.sbk = sbk; o.sbn = sbn;
  o.c = c; o.scb = scb; o.alpha = alpha;
  return o;
}
static hipError_t gemm32_set(int nprob, int batch, int M, int N, int Kd, const GemmSet& set, hipStream_t s) {
  dim3 grid((N + 63) / 64, (M + 63) / 64, batch * nprob);
  k_gemm32<<<grid, 256, 0, s>>>(M, N, Kd, batch, set);
  return hipGetLastError();
}
hipError_t gemm32(int batch, int M, int N, int Kd, float alpha, const float* a, long long sab, int sam, int sak,
                  const float* b, long long sbb, int sbk, int sbn, float* c, long long scb, hipStream_t s) {
  GemmSet set;
  set.p[0] = set.p[1] = set.p[2] = gemm_operands(alpha, a, sab, sam, sak, b, sbb, sbk, sbn, c, scb);
  return gemm32_set(1, batch, M, N, Kd, set, s);
}

// Row-wise softmax backward on the coarse score matrix, in place:
//   sc  holds scale*Qc.Kc^T  -> becomes Ac  = exp(sc - lse_c[row])
//   dsc holds dOc.Vc^T (dAc) -> becomes dSc = Ac * (dAc - sum_j Ac*dAc)
// One wavefront per row, fixed reduction order.
__global__ __launch_bounds__(256) void k_coarse_softmax_bwd(int rows, int Nc, const float* __restrict__ lse_c,
                                                            float* __restrict__ sc, float* __restrict__ dsc,
                                                            const int32_t* __restrict__ kcnt) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  float* s = sc + (long long)row * Nc;
  float* ds = dsc + (long long)row * Nc;
  const float lse = lse_c[row];
  float dot = 0.f;
  for (int j = lane; j < Nc; j += 64) {
    const float a = (!kcnt || kcnt[j] > 0) ? fast_exp2((s[j] - lse) * kLog2e) : 0.f;  // (a dead key cube: no weight)
    s[j] = a;
    dot = fmaf(a, ds[j], dot);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
  for (int j = lane; j < Nc; j += 64) ds[j] = s[j] * (ds[j] - dot);
}

// Coarse backward: dVc = Ac^T dOc, dQc = scale dSc Kc, dKc = scale dSc^T Qc, for Nq query cubes and Nk
// key cubes (see launch_coarse).  `ac` and `dsc` are [BH,Nq,Nk] scratch.
hipError_t launch_coarse_bwd(int BH, int Nq, int Nk, int d, float scale, const float* qc, const float* kc,
                             const float* vc, const float* lse_c, const float* doc, float* ac, float* dsc, float* dqc,
                             float* dkc, float* dvc, const int32_t* kcnt, hipStream_t s) {
  const long long sq = (long long)Nq * d, sk = (long long)Nk * d, ss = (long long)Nq * Nk;
  hipError_t e;
  GemmSet set;
  // one launch: sc = scale * Qc Kc^T ; dAc = dOc Vc^T
  set.p[0] = gemm_operands(scale, qc, sq, d, 1, kc, sk, 1, d, ac, ss);
  set.p[1] = set.p[2] = gemm_operands(1.f, doc, sq, d, 1, vc, sk, 1, d, dsc, ss);
  if ((e = gemm32_set(2, BH, Nq, Nk, d, set, s)) != hipSuccess) return e;
  k_coarse_softmax_bwd<<<(BH * Nq + 3) / 4, 256, 0, s>>>(BH * Nq, Nk, lse_c, ac, dsc, kcnt);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // dVc[j][e] = sum_c Ac[c][j] dOc[c][e] ; dQc[c][e] = scale sum_j dSc[c][j] Kc[j][e] ;
  // dKc[j][e] = scale sum_c dSc[c][j] Qc[c][e]: one launch when the three have the same shape
  GemmOperands dv_ = gemm_operands(1.f, ac, ss, 1, Nk, doc, sq, d, 1, dvc, sk);
  GemmOperands dq_ = gemm_operands(scale, dsc, ss, Nk, 1, kc, sk, d, 1, dqc, sq);
  GemmOperands dk_ = gemm_operands(scale, dsc, ss, 1, Nk, qc, sq, d, 1, dkc, sk);
  if (Nq == Nk) {
    set.p[0] = dv_, set.p[1] = dq_, set.p[2] = dk_;
    return gemm32_set(3, BH, Nq, d, Nq, set, s);
  }
  set.p[0] = dv_, set.p[1] = set.p[2] = dk_;
  if ((e = gemm32_set(2, BH, Nk, d, Nq, set, s)) != hipSuccess) return e;
  set.p[0] = set.p[1] = set.p[2] = dq_;
  return gemm32_set(1, BH, Nq, d, Nk, set, s);
}

// ---------------------------------------------------------------------------------------------
// Transposed block map (CSR): for every key cube j the ascending list of the query cubes that
// selected it.  Built through a bit matrix so that every step is parallel over the whole grid and
// the result does not depend on any execution order (no float or ordering-sensitive atomics; the
// only atomic is a bitwise OR in LDS):
//   bits[bh][j][w], bit q%32 of word q/32  <-  1 for every (q, j) in the index list
//   row_ptr = exclusive scan over j of popcount(row j)        (a wavefront per row, then one
//                                                               workgroup per (b, h) for the scan)
//   col     = positions of the set bits of row j, ascending   (one wavefront per (b, h, j))
constexpr int kMaxCubes = 4096;  // = 4 entries per thread of the 1024-thread scan

// One workgroup per (b, h, word column w): the 32 query cubes 32w .. 32w+31 OR their bits into a
// per-key word held in LDS, then every key row gets its word w written exactly once (no global
// atomics, nothing to clear beforehand).
// (Nq query cubes, Nrows key rows: Nrows = Nq, or 4 Nq when the lists name key cubes of 16 tokens)
__global__ __launch_bounds__(256) void k_map_bits(int Nq, int Nrows, int K, int W32, const int32_t* __restrict__ idx,
                                                  uint32_t* __restrict__ bits) {
  __shared__ uint32_t word[kMaxCubes];
  const int w = blockIdx.x % W32, tid = threadIdx.x;
  const long long bh = blockIdx.x / W32;
  for (int j = tid; j < Nrows; j += 256) word[j] = 0u;
  __syncthreads();
  const int q_lo = w * 32, nq = min(32, Nq - q_lo);
  const int32_t* my = idx + (bh * Nq + q_lo) * (long long)K;
  for (int e = tid; e < nq * K; e += 256) {
    const int c = my[e];
    if (map_takes(c, Nrows)) atomicOr(&word[c], 1u << (e / K));  // (a caller-supplied list is not trusted)
  }
  __syncthreads();
  for (int j = tid; j < Nrows; j += 256) bits[(bh * Nrows + j) * W32 + w] = word[j];
}

// in-degree of every key cube: one wavefront per (b, h, j), written to row_ptr[bh][j] (scanned next)
__global__ __launch_bounds__(256) void k_map_degree(int Nc, int W32, long long rows, const uint32_t* __restrict__ bits,
                                                    int32_t* __restrict__ row_ptr) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // bh * Nc + j
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const uint32_t* r = bits + row * W32;
  int c = 0;
  for (int w = lane; w < W32; w += 64) c += __popc(r[w]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if (lane == 0) row_ptr[(row / Nc) * (Nc + 1) + row % Nc] = c;
}

// Exclusive scan over 4 * 1024 values, 4 consecutive ones per thread of a 1024-thread workgroup:
// v[i] is replaced by the sum of everything before it; returns the grand total.
__device__ __forceinline__ int block_scan4(int* v, int* wsum, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int sum = v[0] + v[1] + v[2] + v[3];
  int incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  __syncthreads();  // wsum may still be read by a previous call
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  int base = 0, total = 0;
  for (int w = 0; w < 16; ++w) {
    if (w < wave) base += wsum[w];
    total += wsum[w];
  }
  int run = base + incl - sum;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = v[i];
    v[i] = run;
    run += t;
  }
  return total;
}

// sum of one value per thread over a 1024-thread workgroup, returned to every thread
__device__ __forceinline__ int block_sum(int x, int* wsum, int tid) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  __syncthreads();  // wsum may still be read by a previous call
  if ((tid & 63) == 0) wsum[tid >> 6] = x;
  __syncthreads();
  int total = 0;
  for (int w = 0; w < 16; ++w) total += wsum[w];
  return total;
}

// exclusive scan of the in-degrees of one (b, h), in place; row_ptr[Nc] = total.  Also cuts the
// work of the dK/dV pass into items and sorts them by length, longest first (counting sort; the
// order among equal lengths is whatever the LDS atomics give, it only decides which workgroup
// starts when).  An item is a key cube's whole list, or -- for a list longer than the split length
// -- one of ceil(deg / length) nearly equal runs of it; each run of such a SPLIT list accumulates
// fp32 partial dK, dV into a numbered slot, summed afterwards in slot order by k_dkv_reduce, so the
// result does not depend on which workgroup ran when.  The split length of a (b, h) is the smallest
// one, not below `seg_min`, at which the runs of all its long lists fit into the `cap` slots the
// slot buffer holds per (b, h): it depends on the in-degrees alone.
//   order: one 16-byte descriptor (key cube, begin, end of the run in col, slot or -1) per dK/dV
//          workgroup, Nc + cap of them per (b, h); unused ones carry key cube -1
//   split: per (b, h) cap/2 + 1 descriptors: [0] = (number of split lists, 0, 0, 0), then
//          (key cube, first slot, number of slots, 0) per split list, in cube order
// (the body, for the 1024 threads of one workgroup: thread `tid` owns cubes 4*tid .. 4*tid+3, whose
// in-degrees it passes in `deg`; `v` returns where their lists begin.  wsum[16] and hist[kMaxCubes] are
// LDS scratch: bucket x of hist counts the items of length Nc - x (the last bucket also takes what
// lies beyond it), then holds the next free slot of the bucket)
__device__ __forceinline__ void map_scan_body(int Nc, int seg_min, int cap, int bh, int tid, const int (&deg)[4], int (&v)[4],
                                              int32_t* __restrict__ row_ptr, int32_t* __restrict__ order,
                                              int32_t* __restrict__ split, int* wsum, int* hist) {
  int32_t* rp = row_ptr + (long long)bh * (Nc + 1);
  const int j0 = tid * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = deg[i];
    hist[j0 + i] = 0;
  }
  const int total = block_scan4(v, wsum, tid);  // (its barriers also cover the clearing of hist)
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (j0 + i < Nc) rp[j0 + i] = v[i];
  if (tid == 0) rp[Nc] = total;

  // the split length: slots_wanted is non-increasing in it and 0 at Nc (no list is longer than Nc)
  auto wanted = [&](int len) {
    int w = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) w += slots_wanted(deg[i], len);
    return block_sum(w, wsum, tid);
  };
  int seg = seg_min;
  if (wanted(seg) > cap) {
    int lo = seg, hi = max(Nc, seg + 1);  // wanted(lo) > cap >= wanted(hi)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (wanted(mid) <= cap) hi = mid; else lo = mid;
    }
    seg = hi;
  }
  // which lists are split, and into how many runs
  int nseg[4], slot[4], rank[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    nseg[i] = split_runs(deg[i], seg);
    slot[i] = nseg[i] > 1 ? nseg[i] : 0;
  }
  block_scan4(slot, wsum, tid);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (nseg[i] > 1 && !split_granted(nseg[i], slot[i], cap)) nseg[i] = 1;
    rank[i] = nseg[i] > 1 ? 1 : 0;
  }
  const int nsplit = block_scan4(rank, wsum, tid);
  int4* sp = (int4*)split + (long long)bh * (cap / 2 + 1);
  if (tid == 0) sp[0] = make_int4(nsplit, 0, 0, 0);
  int extra[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (nseg[i] > 1) sp[1 + rank[i]] = make_int4(j0 + i, slot[i], nseg[i], 0);
    extra[i] = nseg[i] - 1;
  }
  const int items = Nc + block_scan4(extra, wsum, tid);

  // counting sort of the items by length, descending
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (j0 + i < Nc)
      for (int r = 0; r < nseg[i]; ++r) {
        const int len = run_bound(deg[i], nseg[i], r + 1) - run_bound(deg[i], nseg[i], r);
        atomicAdd(&hist[min(Nc - len, kMaxCubes - 1)], 1);
      }
  __syncthreads();
  int first[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) first[i] = hist[j0 + i];
  block_scan4(first, wsum, tid);
#pragma unroll
  for (int i = 0; i < 4; ++i) hist[j0 + i] = first[i];
  __syncthreads();
  int4* ord = (int4*)order + (long long)bh * (Nc + cap);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (j0 + i < Nc)
      for (int r = 0; r < nseg[i]; ++r) {
        const int lo = run_bound(deg[i], nseg[i], r), hi = run_bound(deg[i], nseg[i], r + 1);
        ord[atomicAdd(&hist[min(Nc - (hi - lo), kMaxCubes - 1)], 1)] =
            make_int4(j0 + i, v[i] + lo, v[i] + hi, nseg[i] > 1 ? slot[i] + r : -1);
      }
  for (int e = items + tid; e < Nc + cap; e += 1024) ord[e] = make_int4(-1, 0, 0, -1);
}

__global__ __launch_bounds__(1024) void k_map_scan(int Nc, int seg_min, int cap, int32_t* __restrict__ row_ptr,
                                                   int32_t* __restrict__ order, int32_t* __restrict__ split) {
  __shared__ int wsum[16];
  __shared__ int hist[kMaxCubes];
  const int bh = blockIdx.x, tid = threadIdx.x;
  const int32_t* rp = row_ptr + (long long)bh * (Nc + 1);
  int deg[4], v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) deg[i] = (4 * tid + i < Nc) ? rp[4 * tid + i] : 0;
  map_scan_body(Nc, seg_min, cap, bh, tid, deg, v, row_ptr, order, split, wsum, hist);
}

// the list of key cube j: positions of the set bits of its row `r` (W32 words, global memory or LDS),
// ascending, written to cl[base ..]; one wavefront per row
__device__ __forceinline__ void map_fill_row(const uint32_t* r, int W32, int base, int32_t* __restrict__ cl, int lane) {
  for (int w0 = 0; w0 < W32; w0 += 64) {
    uint32_t word = (w0 + lane < W32) ? r[w0 + lane] : 0u;
    const int c = __popc(word);
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    int pos = base + incl - c;
    while (word) {
      const int b = __ffs(word) - 1;
      cl[pos++] = (w0 + lane) * 32 + b;
      word &= word - 1;
    }
    base += __shfl(incl, 63);
  }
}
__global__ __launch_bounds__(256) void k_map_fill(int Nc, int W32, long long rows, const uint32_t* __restrict__ bits,
                                                  const int32_t* __restrict__ row_ptr, int32_t* __restrict__ col,
                                                  long long col_stride) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // bh * Nc + j
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const long long bh = row / Nc;
  map_fill_row(bits + row * W32, W32, row_ptr[bh * (Nc + 1) + row % Nc], col + bh * col_stride, lane);
}

// Lists that name key cubes of 16 tokens (Sec. 3.2, the 64 x 16 row of the tile-size tables): the bit
// matrix has one row per key cube, four per 64-row key block.  The dK/dV pass works on key blocks, so
// the list of block j is the union of its four rows, and every entry carries, above the query block
// number (bits 16..19), which of the four key cubes that query block selected.
__global__ __launch_bounds__(256) void k_map_degree_sub(int Nc, int W32, long long rows, const uint32_t* __restrict__ bits,
                                                        int32_t* __restrict__ row_ptr) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // bh * Nc + j
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const uint32_t* r = bits + row * 4 * W32;
  int c = 0;
  for (int w = lane; w < W32; w += 64) c += __popc(r[w] | r[W32 + w] | r[2 * W32 + w] | r[3 * W32 + w]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
  if (lane == 0) row_ptr[(row / Nc) * (Nc + 1) + row % Nc] = c;
}
__global__ __launch_bounds__(256) void k_map_fill_sub(int Nc, int W32, long long rows, const uint32_t* __restrict__ bits,
                                                      const int32_t* __restrict__ row_ptr, int32_t* __restrict__ col,
                                                      long long col_stride) {
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // bh * Nc + j
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const long long bh = row / Nc;
  const uint32_t* r = bits + row * 4 * W32;
  int32_t* cl = col + bh * col_stride;
  int base = row_ptr[bh * (Nc + 1) + row % Nc];
  for (int w0 = 0; w0 < W32; w0 += 64) {
    uint32_t u[4] = {0u, 0u, 0u, 0u};
    if (w0 + lane < W32) {
#pragma unroll
      for (int x = 0; x < 4; ++x) u[x] = r[x * W32 + w0 + lane];
    }
    uint32_t word = u[0] | u[1] | u[2] | u[3];
    const int c = __popc(word);
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    int pos = base + incl - c;
    while (word) {
      const int b = __ffs(word) - 1;
      const uint32_t sel = ((u[0] >> b) & 1u) | (((u[1] >> b) & 1u) << 1) | (((u[2] >> b) & 1u) << 2) | (((u[3] >> b) & 1u) << 3);
      cl[pos++] = (int32_t)(((w0 + lane) * 32 + b) | (sel << 16));
      word &= word - 1;
    }
    base += __shfl(incl, 63);
  }
}

// The whole map of one (b, h) in ONE launch, for short sequences (the bit matrix of a (b, h) fits in LDS
// up to kMapOneLaunchMaxCubes key cubes): the four steps above by the 1024 threads of one workgroup --
// bits OR-ed into LDS, in-degrees, scan and work items, lists -- instead of four launches.
constexpr int kMapOneLaunchMaxCubes = 384;  // (measured: ahead of the four launches up to here, level at 512)
__global__ __launch_bounds__(1024) void k_map_one_launch(int Nc, int K, int W32, int seg_min, int cap,
                                                         const int32_t* __restrict__ idx, int32_t* __restrict__ row_ptr,
                                                         int32_t* __restrict__ col, long long col_stride,
                                                         int32_t* __restrict__ order, int32_t* __restrict__ split) {
  __shared__ uint32_t bits_l[kMapOneLaunchMaxCubes * (kMapOneLaunchMaxCubes / 32 + 1)];
  const int WS = W32 | 1;  // odd row stride: the rows the OR step and the count step touch together fall into different banks
  __shared__ int deg_l[kMaxCubes], start_l[kMaxCubes];
  __shared__ int wsum[16];
  __shared__ int hist[kMaxCubes];
  const int bh = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < Nc * WS; i += 1024) bits_l[i] = 0u;
  __syncthreads();
  const int32_t* my = idx + (long long)bh * Nc * K;
  for (int e0 = tid; e0 < Nc * K; e0 += 8 * 1024) {  // (eight loads in flight per thread, then their bits)
    int c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = e0 + u * 1024 < Nc * K ? my[e0 + u * 1024] : -1;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int q = (e0 + u * 1024) / K;
      if (map_takes(c[u], Nc)) atomicOr(&bits_l[c[u] * WS + (q >> 5)], 1u << (q & 31));  // (a caller-supplied list is not trusted)
    }
  }
  __syncthreads();
  for (int j = tid; j < kMaxCubes; j += 1024) {
    int c = 0;
    if (j < Nc)
      for (int w = 0; w < W32; ++w) c += __popc(bits_l[j * WS + w]);
    deg_l[j] = c;
  }
  __syncthreads();
  int deg[4], v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) deg[i] = deg_l[4 * tid + i];
  map_scan_body(Nc, seg_min, cap, bh, tid, deg, v, row_ptr, order, split, wsum, hist);
#pragma unroll
  for (int i = 0; i < 4; ++i) start_l[4 * tid + i] = v[i];
  __syncthreads();
  // lists: one thread per word of the bit matrix (a row has at most 12 words here, so the count of the
  // bits before a word is a short loop over LDS)
  int32_t* cl = col + bh * col_stride;
  for (int i = tid; i < Nc * W32; i += 1024) {
    const int j = i / W32, w = i - j * W32;
    uint32_t word = bits_l[j * WS + w];
    if (!word) continue;
    int pos = start_l[j];
    for (int x = 0; x < w; ++x) pos += __popc(bits_l[j * WS + x]);
    while (word) {
      cl[pos++] = w * 32 + __ffs(word) - 1;
      word &= word - 1;
    }
  }
}

hipError_t launch_transpose_map(int BH, int Nc, int K, const int32_t* idx, uint32_t* bits, int32_t* row_ptr,
                                int32_t* col, int32_t* order, int32_t* split, int seg, int cap, int key_cubes_16,
                                hipStream_t s) {
  const int W32 = (Nc + 31) / 32;
  const long long rows = (long long)BH * Nc;
  hipError_t e;
  if (key_cubes_16) {  // K entries per query block, each a key cube of 16 tokens; bits is [BH, 4 Nc, W32]
    k_map_bits<<<(unsigned)(BH * W32), 256, 0, s>>>(Nc, 4 * Nc, K, W32, idx, bits);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    k_map_degree_sub<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(Nc, W32, rows, bits, row_ptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    k_map_scan<<<BH, 1024, 0, s>>>(Nc, seg, cap, row_ptr, order, split);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    k_map_fill_sub<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(Nc, W32, rows, bits, row_ptr, col, (long long)Nc * K);
    return hipGetLastError();
  }
  if (Nc <= kMapOneLaunchMaxCubes) {
    k_map_one_launch<<<BH, 1024, 0, s>>>(Nc, K, W32, seg, cap, idx, row_ptr, col, (long long)Nc * K, order, split);
    return hipGetLastError();
  }
  k_map_bits<<<(unsigned)(BH * W32), 256, 0, s>>>(Nc, Nc, K, W32, idx, bits);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_map_degree<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(Nc, W32, rows, bits, row_ptr);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_map_scan<<<BH, 1024, 0, s>>>(Nc, seg, cap, row_ptr, order, split);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_map_fill<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(Nc, W32, rows, bits, row_ptr, col, (long long)Nc * K);
  return hipGetLastError();
}

}  // namespace vsa
