// C ABI of libvsa.so: argument validation, workspace carving and kernel sequencing.
// See include/vsa.h for the contract of every entry point.
#include "../../include/vsa.h"

#include <atomic>
#include <vector>

#include "list_rules.h"

#include "vsa_kernels.h"

// Scratch of vsa_forward_static (see there): part of the library's code object, one copy per GPU.
constexpr size_t kStaticScratchBytes = (size_t)VSA_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using vsa::Geo;

constexpr size_t kAlign = 256;
constexpr int kCoarseOneLaunchMaxCubes = 768;  // measured: faster up to the 624 cubes of the 480p shape, slower at 1440
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int check_params(const vsa_params_t* p, Geo* g) {
  if (!p) return VSA_ERR_NULL;
  if (p->B < 1 || p->H < 1 || p->T < 1 || p->Hh < 1 || p->W < 1 || p->Ct < 1 || p->Ch < 1 || p->Cw < 1 || p->d < 1)
    return VSA_ERR_BAD_ARG;
  const long long vol = (long long)p->Ct * p->Ch * p->Cw;
  if (vol != 64 && vol != 128 && vol != 256) return VSA_ERR_UNSUPPORTED;
  if (p->d != 64 && p->d != 128) return VSA_ERR_UNSUPPORTED;
  // pad keys are removed by a bias of -30000 on their raw logits: below this scale the bias, once
  // scaled, no longer drives exp2 to zero against every admissible logit
  if (p->softmax_scale > 0.f && p->softmax_scale < VSA_MIN_SOFTMAX_SCALE) return VSA_ERR_BAD_ARG;
  if (p->softmax_scale != p->softmax_scale) return VSA_ERR_BAD_ARG;
  g->T = p->T; g->Hh = p->Hh; g->W = p->W;
  g->Ct = p->Ct; g->Ch = p->Ch; g->Cw = p->Cw;
  g->Nt = (p->T + p->Ct - 1) / p->Ct;
  g->Nh = (p->Hh + p->Ch - 1) / p->Ch;
  g->Nw = (p->W + p->Cw - 1) / p->Cw;
  long long nc = (long long)g->Nt * g->Nh * g->Nw;
  g->V = (int)vol;
  g->m = (int)(vol / vsa::kTile);
  if (nc * g->m > VSA_MAX_CUBES) return VSA_ERR_UNSUPPORTED;
  long long L = (long long)p->T * p->Hh * p->W;
  g->Nc = (int)nc;
  g->Nb = (int)(nc * g->m);
  g->L = (int)L;
  g->Np = nc * vol;
  if ((long long)p->B * p->H * g->Nb > 0x7fffffffLL / 4) return VSA_ERR_UNSUPPORTED;  // grid sizes stay in 32 bits
  if ((long long)p->B * p->H * g->Nb * p->topk * g->m > 0x7fffffffLL / 2) return VSA_ERR_UNSUPPORTED;
  return VSA_OK;
}

// Coarse stage as one launch (1) or three (0): the caller's flag, else the faster form for the shape.
int coarse_form(const vsa_params_t* p, const Geo& g) {
  if (p->flags & VSA_FLAG_COARSE_UNFUSED) return 0;
  if (p->flags & VSA_FLAG_COARSE_FUSED) return 1;
  return g.Nc <= kCoarseOneLaunchMaxCubes ? 1 : 0;
}

// Mismatched granularity (VSA_FLAG_SELECT_POOLED_2X2): the lists name tiles of (1,2,2) cubes.
bool pooled_select(const vsa_params_t* p) { return (p->flags & VSA_FLAG_SELECT_POOLED_2X2) != 0; }
int list_rows(const vsa_params_t* p, const Geo& g) { return pooled_select(p) ? g.Nc / 4 : g.Nc; }  // rows of block_idx per (b,h)
int blocks_per_entry(const vsa_params_t* p, const Geo& g) { return pooled_select(p) ? 4 : g.m; }    // 64-row blocks a list entry stands for

// Key cubes of 16 tokens (VSA_FLAG_KEY_CUBES_16): four per cube, the lists name them.
bool key16(const vsa_params_t* p) { return (p->flags & VSA_FLAG_KEY_CUBES_16) != 0; }
int key_rows(const vsa_params_t* p, const Geo& g) { return key16(p) ? 4 * g.Nc : g.Nc;  }  // key cubes of the coarse stage

int check_topk(const vsa_params_t* p, const Geo& g) {
  if (pooled_select(p) && (g.m != 1 || g.Nh % 2 || g.Nw % 2)) return VSA_ERR_UNSUPPORTED;
  if (key16(p)) {
    if (pooled_select(p) || p->Ct != 4 || p->Ch != 4 || p->Cw != 4 || 4 * g.Nc > VSA_MAX_CUBES) return VSA_ERR_UNSUPPORTED;
    // a (2,4,2) box of the padded grid is live iff its first token lies inside the valid grid
    const long long live = (long long)((p->T + 1) / 2) * ((p->Hh + 3) / 4) * ((p->W + 1) / 2);
    return (p->topk < 1 || p->topk > live) ? VSA_ERR_BAD_ARG : VSA_OK;
  }
  return (p->topk < 1 || p->topk > list_rows(p, g)) ? VSA_ERR_BAD_ARG : VSA_OK;
}

bool misaligned(const void* ptr) { return ptr && ((uintptr_t)ptr & 15u); }

float scale_of(const vsa_params_t* p) { return p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d); }

// Bump allocator over the caller's workspace.
struct Carver {
  unsigned char* base;
  size_t used = 0;
  explicit Carver(void* b) : base((unsigned char*)b) {}
  template <typename T>
  T* take(size_t count) {
    T* r = (T*)(base + used);
    used += align_up(count * sizeof(T));
    return r;
  }
};

struct FwdWs {
  uint64_t* mask;
  int32_t* kcnt;
  float *qc, *kc, *vc, *oc, *lse_c, *sc, *ps;
  int32_t *idx, *idx_blocks;
  size_t bytes;
};
FwdWs carve_fwd(const vsa_params_t* p, const Geo& g, void* ws) {
  Carver c(ws);
  size_t bh = (size_t)p->B * p->H;
  FwdWs w;
  const size_t nk = (size_t)key_rows(p, g);
  w.mask = c.take<uint64_t>(g.Nb);
  w.kcnt = key16(p) ? c.take<int32_t>(nk) : nullptr;
  w.qc = c.take<float>(bh * g.Nc * p->d);
  w.kc = c.take<float>(bh * nk * p->d);
  w.vc = c.take<float>(bh * nk * p->d);
  w.oc = c.take<float>(bh * g.Nc * p->d);
  w.lse_c = c.take<float>(bh * g.Nc);
  const size_t bpe = (size_t)blocks_per_entry(p, g), rows = (size_t)list_rows(p, g);
  w.idx = c.take<int32_t>(bh * rows * p->topk);
  w.sc = c.take<float>(bh * g.Nc * nk);
  w.idx_blocks = bpe > 1 ? c.take<int32_t>(bh * g.Nb * p->topk * bpe) : nullptr;
  w.ps = pooled_select(p) ? c.take<float>(bh * rows * rows) : nullptr;
  w.bytes = c.used;
  return w;
}

struct BwdWs {
  uint64_t* mask;
  int32_t* kcnt;
  float *qc, *kc, *vc, *ld, *doc, *ac, *dsc, *dqc, *dkc, *dvc;
  void *dof, *ldb;
  int32_t *row_ptr, *col, *order, *split, *idx_blocks;
  uint32_t* bits;
  float* parts;
  int seg, cap;
  size_t bytes;
};
// How the dK/dV pass cuts long transposed lists (see k_map_scan): a list longer than `seg` entries
// is worked off by several workgroups; at most `cap` partial-result slots per (b, h).  `seg` is the
// smallest split length: it aims at items no longer than half of what a compute unit gets when the
// work is spread evenly (256 units), but not so short that start-up and the extra pass over the
// partial sums outweigh the gain; the map scan lengthens it per (b, h) until the slots suffice.
void split_plan(const vsa_params_t* p, const Geo& g, int* seg, int* cap) {
  const long long kb = (long long)p->topk * blocks_per_entry(p, g);  // list length in blocks
  const long long entries = (long long)p->B * p->H * g.Nb * kb;
  long long s = entries / 512;
  if (s > 4 * kb) s = 4 * kb;
  if (s < 16) s = 16;
  *seg = (int)s;
  int c = g.Nb / 4;
  *cap = c < 16 ? 16 : (c > 64 ? 64 : c);
}
BwdWs carve_bwd(const vsa_params_t* p, const Geo& g, void* ws) {
  Carver c(ws);
  size_t bh = (size_t)p->B * p->H;
  BwdWs w;
  const size_t kb = (size_t)p->topk * blocks_per_entry(p, g);
  const size_t nk = (size_t)key_rows(p, g);
  w.mask = c.take<uint64_t>(g.Nb);
  w.kcnt = key16(p) ? c.take<int32_t>(nk) : nullptr;
  w.qc = c.take<float>(bh * g.Nc * p->d);
  w.kc = c.take<float>(bh * nk * p->d);
  w.vc = c.take<float>(bh * nk * p->d);
  w.ld = c.take<float>(2 * bh * g.Np);
  w.ldb = c.take<uint32_t>(4 * bh * g.Np);
  w.doc = c.take<float>(bh * g.Nc * p->d);
  w.ac = c.take<float>(bh * g.Nc * nk);
  w.dsc = c.take<float>(bh * g.Nc * nk);
  w.dqc = c.take<float>(bh * g.Nc * p->d);
  w.dkc = c.take<float>(bh * nk * p->d);
  w.dvc = c.take<float>(bh * nk * p->d);
  w.dof = c.take<uint16_t>(bh * g.Np * p->d);
  w.row_ptr = c.take<int32_t>(bh * (g.Nb + 1));
  w.col = c.take<int32_t>(bh * g.Nb * kb);
  w.bits = c.take<uint32_t>(bh * (key16(p) ? 4 : 1) * g.Nb * ((g.Nb + 31) / 32));
  w.idx_blocks = blocks_per_entry(p, g) > 1 ? c.take<int32_t>(bh * g.Nb * kb) : nullptr;
  split_plan(p, g, &w.seg, &w.cap);
  w.order = c.take<int32_t>(4 * bh * (g.Nb + w.cap));  // (block, run begin, run end, slot) per dK/dV workgroup
  w.split = c.take<int32_t>(4 * bh * (w.cap / 2 + 1));
  w.parts = c.take<float>(bh * w.cap * 2 * vsa::kTile * p->d);
  w.bytes = c.used;
  return w;
}

// Optional per-kernel timing (vsa_profile_*): events are created up front by vsa_profile_begin,
// so a profiled call still allocates nothing.  One global recorder, not thread-safe.
struct Profiler {
  bool on = false;
  int cap = 0, n = 0;
  hipEvent_t* start = nullptr;
  hipEvent_t* stop = nullptr;
  const char** name = nullptr;
} g_prof;

struct Timed {
  int slot = -1;
  hipStream_t s;
  Timed(const char* name, hipStream_t stream) : s(stream) {
    if (g_prof.on && g_prof.n < g_prof.cap) {
      slot = g_prof.n++;
      g_prof.name[slot] = name;
      (void)hipEventRecord(g_prof.start[slot], s);
    }
  }
  ~Timed() {
    if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s);
  }
};

#define VSA_TRY(name, expr)                \
  do {                                     \
    Timed timed_(name, s);                 \
    if ((expr) != hipSuccess) return VSA_ERR_HIP; \
  } while (0)

int check_forward_args(const vsa_params_t* p, Geo* g, const void* q, const void* k, const void* v, const void* gate_c,
                       const void* gate_f, const void* out, const int32_t* block_idx, const void* out_fine,
                       const float* lse_fine, const float* out_coarse, const float* lse_coarse) {
  int rc = check_params(p, g);
  if (rc != VSA_OK) return rc;
  if ((rc = check_topk(p, *g)) != VSA_OK) return rc;
  const bool given = (p->flags & VSA_FLAG_INDICES_GIVEN) != 0;
  if (!q || !k || !v || !gate_c || !out || (given && !block_idx)) return VSA_ERR_NULL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(gate_c) || misaligned(gate_f) || misaligned(out) ||
      misaligned(block_idx) || misaligned(out_fine) || misaligned(lse_fine) || misaligned(out_coarse) ||
      misaligned(lse_coarse))
    return VSA_ERR_ALIGN;
  return VSA_OK;
}

// The forward's kernel sequence on validated arguments; `workspace` holds at least carve_fwd().bytes.
int enqueue_forward(const vsa_params_t* p, const Geo& g, const void* q, const void* k, const void* v,
                    const void* gate_c, const void* gate_f, void* out, int32_t* block_idx, void* out_fine,
                    float* lse_fine, float* out_coarse, float* lse_coarse, void* workspace, hipStream_t s) {
  const bool given = (p->flags & VSA_FLAG_INDICES_GIVEN) != 0;
  FwdWs w = carve_fwd(p, g, workspace);
  const int BH = p->B * p->H;
  const float scale = scale_of(p);
  float* oc = out_coarse ? out_coarse : w.oc;
  float* lse_c = lse_coarse ? lse_coarse : w.lse_c;
  int32_t* idx = block_idx ? block_idx : w.idx;

  const bool sub = key16(p);
  VSA_TRY("pool", vsa::launch_pool(g, BH, p->d, w.mask, q, k, v, w.qc, w.kc, w.vc, sub ? 1 : 3, s));
  if (sub) VSA_TRY("pool", vsa::launch_pool_keys16(BH, g.Nc, p->d, w.mask, w.kcnt, k, v, w.kc, w.vc, s));
  const bool pooled = pooled_select(p);
  VSA_TRY("coarse", vsa::launch_coarse(BH, g.Nc, key_rows(p, g), p->d, p->topk, scale, w.qc, w.kc, w.vc, w.sc, oc, lse_c, idx,
                            (given || pooled) ? 0 : 1, (pooled || sub) ? 0 : coarse_form(p, g), w.kcnt, s));
  // the fine stage works on 64-row blocks: a cube of m blocks contributes m list entries, a tile of
  // (1,2,2) cubes its four cubes
  const int32_t* lists = idx;
  if (pooled) {
    if (!given) VSA_TRY("pooled_select", vsa::launch_pooled_select(BH, g.Nt, g.Nh, g.Nw, p->topk, w.sc, w.ps, idx, s));
    VSA_TRY("expand_lists", vsa::launch_expand_tiles(BH, g.Nt, g.Nh, g.Nw, p->topk, idx, w.idx_blocks, s));
    lists = w.idx_blocks;
  } else if (g.m > 1) {
    VSA_TRY("expand_lists", vsa::launch_expand_lists(BH, g.Nc, p->topk, g.m, idx, w.idx_blocks, s));
    lists = w.idx_blocks;
  }
  VSA_TRY("fine_fwd", vsa::launch_fine_fwd(BH, g.Nb, p->d, p->topk * blocks_per_entry(p, g), scale, q, k, v, gate_c, gate_f, lists, oc, w.mask, out,
                               out_fine, lse_fine, p->H, (p->flags & VSA_FLAG_OUT_TOKEN_MAJOR) ? 1 : 0, g.m, sub ? 1 : 0, s));
  return VSA_OK;
}

// Scratch of vsa_forward_static: device memory that belongs to the library's code object, one copy
// per GPU at that GPU's own address, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress -- never a device address -- so every use goes through the
// pointer looked up once per device (with that device current) and kept here.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

void* static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    // two threads may both look it up: they get the same address
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  return ptr;
}

}  // namespace

extern "C" {

int vsa_padded_tokens(const vsa_params_t* p, int64_t* Np, int32_t* Nc) {
  Geo g;
  int rc = check_params(p, &g);
  if (rc != VSA_OK) return rc;
  if (Np) *Np = g.Np;
  if (Nc) *Nc = g.Nc;
  return VSA_OK;
}

size_t vsa_workspace_bytes(const vsa_params_t* p, int backward) {
  Geo g;
  if (check_params(p, &g) != VSA_OK || check_topk(p, g) != VSA_OK) return 0;
  return backward ? carve_bwd(p, g, nullptr).bytes : carve_fwd(p, g, nullptr).bytes;
}

int vsa_tile_permute(const vsa_params_t* p, const void* src, void* dst, int inverse, void* hip_stream) {
  Geo g;
  int rc = check_params(p, &g);
  if (rc != VSA_OK) return rc;
  if (!src || !dst) return VSA_ERR_NULL;
  if (misaligned(src) || misaligned(dst)) return VSA_ERR_ALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  VSA_TRY("tile_permute", vsa::launch_tile_permute(g, p->B * p->H, (p->flags & VSA_FLAG_RASTER_BLHD) ? p->H : 0, p->d, src, dst, inverse != 0, s));
  return VSA_OK;
}

int vsa_forward(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                const void* gate_f, void* out, int32_t* block_idx, void* out_fine, float* lse_fine,
                float* out_coarse, float* lse_coarse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Geo g;
  int rc = check_forward_args(p, &g, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse, lse_coarse);
  if (rc != VSA_OK) return rc;
  if (misaligned(workspace)) return VSA_ERR_ALIGN;
  if (!workspace || workspace_bytes < carve_fwd(p, g, nullptr).bytes) return VSA_ERR_WORKSPACE;
  return enqueue_forward(p, g, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse, lse_coarse,
                         workspace, (hipStream_t)hip_stream);
}

size_t vsa_static_scratch_bytes(void) { return kStaticScratchBytes; }

int vsa_forward_static(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                       const void* gate_f, void* out, int32_t* block_idx, void* out_fine, float* lse_fine,
                       float* out_coarse, float* lse_coarse, void* hip_stream) {
  Geo g;
  int rc = check_forward_args(p, &g, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse, lse_coarse);
  if (rc != VSA_OK) return rc;
  if (carve_fwd(p, g, nullptr).bytes > kStaticScratchBytes) return VSA_ERR_SCRATCH_LIMIT;
  void* ws = static_scratch_of_current_device();
  if (!ws) return VSA_ERR_HIP;
  return enqueue_forward(p, g, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse, lse_coarse, ws,
                         (hipStream_t)hip_stream);
}

int vsa_backward(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                 const void* gate_f, const void* dout, const int32_t* block_idx, const void* out_fine,
                 const float* lse_fine, const float* out_coarse, const float* lse_coarse, void* dq, void* dk,
                 void* dv, void* dgate_c, void* dgate_f, void* workspace, size_t workspace_bytes,
                 void* hip_stream) {
  Geo g;
  int rc = check_params(p, &g);
  if (rc != VSA_OK) return rc;
  if ((rc = check_topk(p, g)) != VSA_OK) return rc;
  if (!q || !k || !v || !gate_c || !dout || !block_idx || !out_fine || !lse_fine || !out_coarse || !lse_coarse ||
      !dq || !dk || !dv || !dgate_c)
    return VSA_ERR_NULL;
  if ((gate_f == nullptr) != (dgate_f == nullptr)) return VSA_ERR_BAD_ARG;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(gate_c) || misaligned(gate_f) ||
      misaligned(dout) || misaligned(block_idx) || misaligned(out_fine) || misaligned(lse_fine) ||
      misaligned(out_coarse) || misaligned(lse_coarse) || misaligned(dq) || misaligned(dk) || misaligned(dv) ||
      misaligned(dgate_c) || misaligned(dgate_f) || misaligned(workspace))
    return VSA_ERR_ALIGN;
  if (!workspace || workspace_bytes < carve_bwd(p, g, nullptr).bytes) return VSA_ERR_WORKSPACE;

  hipStream_t s = (hipStream_t)hip_stream;
  BwdWs w = carve_bwd(p, g, workspace);
  const int BH = p->B * p->H;
  const float scale = scale_of(p);

  // forward and backward carve the cube masks and the pooled tensors at the same offsets
  const bool sub = key16(p);
  if (!(p->flags & VSA_FLAG_WORKSPACE_KEPT)) {
    VSA_TRY("pool", vsa::launch_pool(g, BH, p->d, w.mask, q, k, v, w.qc, w.kc, w.vc, sub ? 1 : 3, s));
    if (sub) VSA_TRY("pool", vsa::launch_pool_keys16(BH, g.Nc, p->d, w.mask, w.kcnt, k, v, w.kc, w.vc, s));
  }
  VSA_TRY("bwd_pre", vsa::launch_bwd_pre(BH, g.Nc, g.m, p->d, w.mask, dout, gate_c, gate_f, out_fine, out_coarse, dgate_c, dgate_f,
                              w.dof, w.ld, w.ldb, scale, w.doc, lse_fine, p->H, (p->flags & VSA_FLAG_OUT_TOKEN_MAJOR) ? 1 : 0, s));
  VSA_TRY("coarse_bwd", vsa::launch_coarse_bwd(BH, g.Nc, key_rows(p, g), p->d, scale, w.qc, w.kc, w.vc, lse_coarse, w.doc, w.ac, w.dsc,
                                 w.dqc, w.dkc, w.dvc, w.kcnt, s));
  const int32_t* lists = block_idx;
  const int kb = p->topk * blocks_per_entry(p, g);
  if (pooled_select(p)) {
    VSA_TRY("expand_lists", vsa::launch_expand_tiles(BH, g.Nt, g.Nh, g.Nw, p->topk, block_idx, w.idx_blocks, s));
    lists = w.idx_blocks;
  } else if (g.m > 1) {
    VSA_TRY("expand_lists", vsa::launch_expand_lists(BH, g.Nc, p->topk, g.m, block_idx, w.idx_blocks, s));
    lists = w.idx_blocks;
  }
  VSA_TRY("transpose_map", vsa::launch_transpose_map(BH, g.Nb, kb, lists, w.bits, w.row_ptr, w.col, w.order, w.split, w.seg, w.cap, sub ? 1 : 0, s));
  VSA_TRY("fine_bwd_dq", vsa::launch_fine_bwd_dq(BH, g.Nb, p->d, kb, scale, q, k, v, w.dof, lists, w.ld,
                                  w.dqc, w.mask, dq, g.m, sub ? 1 : 0, s));
  VSA_TRY("fine_bwd_dkv", vsa::launch_fine_bwd_dkv(BH, g.Nb, p->d, kb, scale, q, k, v, w.dof, w.col, w.order, w.split, w.parts,
                                   w.cap, w.ldb, w.dkc, w.dvc, w.mask, dk, dv, g.m, sub ? 1 : 0, s));
  return VSA_OK;
}

int vsa_host_replay_lists(const vsa_params_t* p, const int32_t* host_block_idx, int64_t* report) {
  Geo g;
  int rc = check_params(p, &g);
  if (rc != VSA_OK) return rc;
  if ((rc = check_topk(p, g)) != VSA_OK) return rc;
  if (!host_block_idx) return VSA_ERR_NULL;
  // the kernels see lists of 64-row blocks: a cube of m blocks expands to m entries
  const int Nc = g.Nb, bpe = blocks_per_entry(p, g), K = p->topk * bpe;
  int seg_min, cap;
  split_plan(p, g, &seg_min, &cap);
  std::vector<int32_t> expanded((size_t)Nc * K);
  int64_t bad = 0, max_deg = 0, max_items = 0, max_slots = 0, max_split = 0, max_col = 0;
  std::vector<unsigned char> bit((size_t)Nc * Nc);
  std::vector<int> deg(Nc), beg(Nc);
  for (long long bh = 0; bh < (long long)p->B * p->H; ++bh) {
    for (int row = 0; row < Nc; ++row)
      for (int e = 0; e < K; ++e)
        expanded[(size_t)row * K + e] =
            pooled_select(p)
                ? vsa::tile_member_cube(host_block_idx[(bh * (g.Nc / 4) + vsa::tile_of_cube(row, g.Nh, g.Nw)) * p->topk + e / 4],
                                        e % 4, g.Nt, g.Nh, g.Nw)
                : vsa::expanded_entry(host_block_idx[(bh * g.Nc + row / g.m) * p->topk + e / g.m], g.m, e % g.m);
    const int32_t* lists = expanded.data();
    // key cubes of 16 tokens: an entry names key cube 4*block + s, clamped or skipped against 4*Nc; the
    // fetch starts at the key cube's first slot and reaches at most subcube_slot(15) rows further
    const int per = key16(p) ? 4 : 1;
    // forward and dQ pass: every lane of every 64-entry chunk reads a list slot, then fetches a cube
    for (int c = 0; c < Nc; ++c)
      for (int chunk = 0; chunk * 64 < K; ++chunk)
        for (int lane = 0; lane < 64; ++lane) {
          const int slot = vsa::list_slot(chunk, lane, K);
          if (slot < 0 || slot >= K) { ++bad; continue; }
          const int id = vsa::clamp_cube(lists[(size_t)c * K + slot], per * Nc);
          const int cube = id / per;
          if (id < 0 || cube >= Nc) ++bad;
          if (per == 4 && vsa::subcube_first_slot(id & 3) + vsa::subcube_slot(15) > 63) ++bad;
        }
    // transposed map: one bit per (query cube, key cube) pair that names a cube
    std::fill(bit.begin(), bit.end(), 0);
    for (int c = 0; c < Nc; ++c)
      for (int e = 0; e < K; ++e) {
        const int raw = lists[(size_t)c * K + e];
        if (vsa::map_takes(raw, per * Nc)) {
          if (raw < 0 || raw / per >= Nc) { ++bad; continue; }
          bit[(size_t)(raw / per) * Nc + c] = 1;  // (the dK/dV pass works on the union over a block's key cubes)
        }
      }
    long long total = 0;
    for (int j = 0; j < Nc; ++j) {
      int dsum = 0;
      for (int c = 0; c < Nc; ++c) dsum += bit[(size_t)j * Nc + c];
      deg[j] = dsum;
      beg[j] = (int)total;
      total += dsum;
      if (dsum > max_deg) max_deg = dsum;
    }
    if (total > (long long)Nc * K) ++bad;  // capacity of the col array
    if (total > max_col) max_col = total;
    // split length of this (b, h): the smallest one >= seg_min at which all wanted slots fit
    int seg = seg_min;
    {
      auto wanted_at = [&](int len) {
        long long w = 0;
        for (int j = 0; j < Nc; ++j) w += vsa::slots_wanted(deg[j], len);
        return w;
      };
      while (wanted_at(seg) > cap) ++seg;
    }
    // dK/dV items: whole lists and the runs of split lists
    int wanted = 0, nsplit = 0, items = 0, slots_hi = 0;
    for (int j = 0; j < Nc; ++j) {
      int runs = vsa::split_runs(deg[j], seg);
      const int want = runs > 1 ? runs : 0;
      const bool granted = vsa::split_granted(runs, wanted, cap);
      const int slot0 = wanted;
      wanted += want;
      if (runs > 1 && !granted) ++bad;  // the split length was chosen so that every long list fits
      if (!granted) runs = 1;
      if (runs > 1) {
        ++nsplit;
        if (slot0 < 0 || slot0 + runs > cap) ++bad;
        if (slot0 + runs > slots_hi) slots_hi = slot0 + runs;
      }
      int covered = 0;
      for (int r = 0; r < runs; ++r) {
        const int lo = vsa::run_bound(deg[j], runs, r), hi = vsa::run_bound(deg[j], runs, r + 1);
        if (lo != covered || hi < lo || hi > deg[j]) ++bad;
        covered = hi;
        // the dK/dV workgroup of this run reads col[beg + lo + list_slot(chunk, lane, hi - lo)]
        const int n = hi - lo;
        for (int chunk = 0; chunk * 64 < n; ++chunk)
          for (int lane = 0; lane < 64; ++lane) {
            const long long at = (long long)beg[j] + lo + vsa::list_slot(chunk, lane, n);
            if (at < beg[j] + lo || at >= beg[j] + hi || at >= (long long)Nc * K) ++bad;
          }
        ++items;
      }
      if (covered != deg[j]) ++bad;
    }
    if (items > Nc + cap) ++bad;     // descriptors per (b, h)
    if (nsplit > cap / 2) ++bad;     // entries of the split-list table
    if (items > max_items) max_items = items;
    if (slots_hi > max_slots) max_slots = slots_hi;
    if (nsplit > max_split) max_split = nsplit;
  }
  if (report) {
    report[0] = bad; report[1] = max_deg; report[2] = max_items; report[3] = max_slots;
    report[4] = max_split; report[5] = max_col; report[6] = seg_min; report[7] = cap;
  }
  return bad ? VSA_ERR_BAD_ARG : VSA_OK;
}

int vsa_profile_begin(int max_records) {
  if (g_prof.on || max_records < 1) return VSA_ERR_BAD_ARG;
  g_prof.start = new hipEvent_t[max_records];
  g_prof.stop = new hipEvent_t[max_records];
  g_prof.name = new const char*[max_records];
  for (int i = 0; i < max_records; ++i)
    if (hipEventCreate(&g_prof.start[i]) != hipSuccess || hipEventCreate(&g_prof.stop[i]) != hipSuccess)
      return VSA_ERR_HIP;
  g_prof.cap = max_records;
  g_prof.n = 0;
  g_prof.on = true;
  return VSA_OK;
}

int vsa_profile_count(void) { return g_prof.n; }

const char* vsa_profile_name(int i) { return (i >= 0 && i < g_prof.n) ? g_prof.name[i] : ""; }

float vsa_profile_ms(int i) {
  float ms = -1.f;
  if (i >= 0 && i < g_prof.n && hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) ms = -1.f;
  return ms;
}

int vsa_profile_end(void) {
  if (!g_prof.on) return VSA_ERR_BAD_ARG;
  for (int i = 0; i < g_prof.cap; ++i) {
    (void)hipEventDestroy(g_prof.start[i]);
    (void)hipEventDestroy(g_prof.stop[i]);
  }
  delete[] g_prof.start;
  delete[] g_prof.stop;
  delete[] g_prof.name;
  g_prof = Profiler();
  return VSA_OK;
}

int vsa_bench_mfma_rate(const void* operands, float* sink, int workgroups, int iters, double* flops, void* hip_stream) {
  if (!operands || !sink || !flops) return VSA_ERR_NULL;
  if (workgroups < 1 || iters < 1 || workgroups > (1 << 20) || iters > (1 << 24)) return VSA_ERR_BAD_ARG;
  if (misaligned(operands) || misaligned(sink)) return VSA_ERR_ALIGN;
  *flops = (double)workgroups * 4.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
  return vsa::launch_mfma_rate(operands, sink, workgroups, iters, (hipStream_t)hip_stream) == hipSuccess ? VSA_OK : VSA_ERR_HIP;
}

const char* vsa_status_string(int status) {
  switch (status) {
    case VSA_OK: return "ok";
    case VSA_ERR_NULL: return "a required pointer is NULL";
    case VSA_ERR_BAD_ARG: return "bad argument (dimension or topk out of range, gate_f/dgate_f mismatch)";
    case VSA_ERR_UNSUPPORTED: return "unsupported configuration (cube volume not 64/128/256, d not 64/128, too many cubes)";
    case VSA_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case VSA_ERR_WORKSPACE: return "workspace missing or too small";
    case VSA_ERR_HIP: return "a kernel launch failed";
    case VSA_ERR_SCRATCH_LIMIT: return "the problem needs more scratch than the static buffer of vsa_forward_static holds";
    default: return "unknown status";
  }
}

}  // extern "C"
