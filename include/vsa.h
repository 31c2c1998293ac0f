/*
 * vsa.h -- C ABI of the MI355X (gfx950) Video Sparse Attention library, libvsa.so.
 *
 * Video Sparse Attention (arxiv 2505.13389, Sec. 2.2) replaces dense 3D attention of a
 * video diffusion transformer by two stages over (Ct,Ch,Cw) token cubes ((4,4,4) in the paper's
 * main configuration; Sec. 3.2 ablates larger ones): a
 * coarse stage (mean-pooled cube-level attention that also picks, per query cube, the
 * top-K key cubes) and a fine stage (token-level block-sparse attention over the picked
 * cubes); the output is the gated sum O = O_c * G_c + O_f * G_f.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers (HIP), 16-byte aligned, contiguous, row-major.
 *     `const vsa_params_t*` and the out-parameters of vsa_padded_tokens are HOST pointers.
 *   - The caller owns every buffer.  The library never allocates, frees or synchronises:
 *     calls enqueue kernels on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and return.  Scratch comes from `workspace` (>= vsa_workspace_bytes).
 *   - "raster" order: token (t,h,w) of the valid T x Hh x W grid at n = t*Hh*W + h*W + w
 *     (Sec. 2.1).  "tiled" order: the index equation of Sec. 2.2 on the grid padded up to
 *     cube multiples, Np tokens = Nc cubes x V (V = Ct*Ch*Cw = 64, 128 or 256); each cube is V
 *     consecutive rows.  The attention tile equals the cube: a query cube attends to the whole
 *     of each selected key cube.
 *   - Pad slots (tiled rows outside the valid grid) are defined by geometry alone.  They
 *     are never keys, are excluded from pooled means, and their rows of every output and
 *     gradient are written as zero; whatever finite values the caller stores there in an
 *     input are ignored (NaN or Inf there is not allowed).
 *   - Value range: raw dot products |q . k| of token pairs must stay below 15000 (the pad
 *     keys of a partially filled cube are removed by adding -30000 to their raw logits).
 *   - Results are deterministic (bit-identical across calls on the same inputs).
 *   - Return value: VSA_OK (0) or a negative vsa_status.  Validation errors are detected
 *     before anything is enqueued; VSA_ERR_HIP (a launch rejected by the runtime) can leave
 *     the earlier kernels of that call enqueued.
 */
#ifndef VSA_H_
#define VSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VSA_OK = 0,
  VSA_ERR_NULL = -1,        /* a required pointer is NULL                              */
  VSA_ERR_BAD_ARG = -2,     /* non-positive dimension, topk outside 1..Nc, scale too small */
  VSA_ERR_UNSUPPORTED = -3, /* cube volume not 64/128/256, d not in {64,128}, too many cubes */
  VSA_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned                 */
  VSA_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than vsa_workspace_bytes      */
  VSA_ERR_HIP = -6,         /* a kernel launch was rejected by the runtime             */
  VSA_ERR_SCRATCH_LIMIT = -7 /* vsa_forward_static: the problem needs more scratch than the static buffer */
} vsa_status;

#define VSA_FLAG_INDICES_GIVEN 1u /* vsa_forward: block_idx is an INPUT, top-K is skipped */
#define VSA_FLAG_RASTER_BLHD 2u   /* vsa_tile_permute: the raster tensor is token-major [B,L,H,d] */
#define VSA_FLAG_WORKSPACE_KEPT 4u /* vsa_backward: `workspace` is the buffer the matching vsa_forward
                                      call (same parameters, same q, k, v) was given, and nothing has
                                      written to it since: the pooled tensors it still holds are used
                                      instead of being computed again.  Size it for the backward. */
#define VSA_FLAG_COARSE_FUSED 8u    /* vsa_forward: run the coarse stage as ONE launch that keeps the score block
                                      in LDS (Sec. 2.4, App. D; up to 1536 cubes, ignored above) ...          */
#define VSA_FLAG_COARSE_UNFUSED 64u /* ... or as three launches with the score matrix in the workspace.  With
                                      neither flag the library picks the faster form for the shape.  The two
                                      forms use different matrix instructions: their logits agree to the last
                                      few bits, so their selections can differ on near ties only.            */
#define VSA_FLAG_OUT_TOKEN_MAJOR 16u /* vsa_forward: `out` is written token-major, bf16 [B,Np,H,d] = [B,Np,H*d]
                                       in tiled token order: the layout the output projection consumes
                                       ("b h l d -> b l (h d)", last line of the App. B listing) when
                                       the activations stay tiled across the transformer (App. B caption),
                                       so no relayout pass remains.  vsa_backward: `dout` is read in the
                                       same layout.  All other tensors keep [B,H,Np,d]. */
#define VSA_FLAG_SELECT_POOLED_2X2 32u /* mismatched granularity (Sec. 3.2): the coarse stage pools over the
                                         (Ct,Ch,Cw) cubes (64 tokens), the fine stage attends in tiles of
                                         (1,2,2) cubes = 256 tokens.  The coarse attention map is averaged
                                         over the 2x2 cubes of the query tile and of the key tile, and the
                                         topk largest entries of each row of the pooled map select key
                                         TILES: block_idx is then int32 [B,H,Ns,topk], Ns = Nc/4 tiles,
                                         tile (st,sh,sw) = (st*Nh/2 + sh)*Nw/2 + sw holding cubes
                                         (st, 2sh+a, 2sw+b); 1 <= topk <= Ns.  Needs 64-token cubes and
                                         even numbers of cubes along h and w (else VSA_ERR_UNSUPPORTED).
                                         Pass the flag to vsa_forward, vsa_backward and
                                         vsa_workspace_bytes alike. */
#define VSA_FLAG_KEY_CUBES_16 128u /* the 64 x 16 tiles of the Sec. 3.2 tile-size tables: queries keep the (4,4,4)
                                     cubes (and the tensors their token order), keys are pooled and selected
                                     in the (2,4,2) boxes nested in them.  Key cube 4*c + 2a + b holds the
                                     tokens of cube c with (t mod 4)/2 = a and (w mod 4)/2 = b; Nk = 4*Nc.
                                     topk counts key cubes, 1 <= topk <= live key cubes =
                                     ceil(T/2)*ceil(Hh/4)*ceil(W/2) (a key cube of a padded grid may hold
                                     no valid token: it is left out of the coarse softmax and never
                                     selected); block_idx is int32 [B,H,Nc,topk] of key cube numbers,
                                     ascending.  Needs Ct,Ch,Cw = 4,4,4 and at most VSA_MAX_CUBES/4 cubes;
                                     not together with VSA_FLAG_SELECT_POOLED_2X2; the coarse stage runs
                                     as three launches.  Pass the flag to vsa_forward, vsa_backward and
                                     vsa_workspace_bytes alike. */
#define VSA_MIN_SOFTMAX_SCALE (1.0f / 64.0f) /* smallest explicit softmax_scale accepted (the pad-key bias of
                                               -30000 must still underflow the exponential once scaled) */
#define VSA_MAX_CUBES 4096        /* largest supported Np / 64 (= Nc for 64-token cubes)  */
#define VSA_STATIC_SCRATCH_MIB 40 /* size of the scratch buffer behind vsa_forward_static, MiB */

typedef struct {
  int32_t B, H;        /* batch, heads                                                   */
  int32_t T, Hh, W;    /* valid latent grid in tokens                                    */
  int32_t Ct, Ch, Cw;  /* cube shape; Ct*Ch*Cw must be 64 (Sec. 2.2: (4,4,4)), 128 or 256  */
  int32_t d;           /* head dimension: 64 or 128                                      */
  int32_t topk;        /* key cubes per query cube, 1..Nc; Nc = the dense path           */
  float softmax_scale; /* <= 0 selects 1/sqrt(d) (Sec. 2.1); else >= VSA_MIN_SOFTMAX_SCALE       */
  uint32_t flags;      /* VSA_FLAG_*                                                     */
} vsa_params_t;

/* Padded token count Np and cube count Nc of the grid in `p` (Sec. 2.2: (Nt,Nh,Nw) =
 * ceil(T/Ct), ceil(Hh/Ch), ceil(W/Cw); Np = Ct*Ch*Cw*Nc).  Host-only. */
int vsa_padded_tokens(const vsa_params_t* p, int64_t* Np, int32_t* Nc);

/* Bytes of scratch vsa_forward (backward == 0) or vsa_backward (backward != 0) needs.
 * Returns 0 for invalid parameters.  Host-only. */
size_t vsa_workspace_bytes(const vsa_params_t* p, int backward);

/* Raster <-> tiled token permutation of one bf16 tensor (Sec. 2.2 index equation; App. B
 * tile()/untile()).
 *   inverse == 0: src [B,H,T*Hh*W,d] raster -> dst [B,H,Np,d] tiled, pad rows zero-filled.
 *   inverse != 0: src [B,H,Np,d] tiled -> dst [B,H,T*Hh*W,d] raster, pad rows dropped.
 * With VSA_FLAG_RASTER_BLHD in p->flags the raster tensor (src or dst, by direction) is laid
 * out [B, T*Hh*W, H, d] instead: the layout of the projections around the attention
 * ("b h l d <-> b l (h d)" at both ends of the App. B listing), so that the head transpose
 * rides on the permutation instead of costing a pass of its own.  The tiled side is unchanged.
 * src and dst must not overlap. */
int vsa_tile_permute(const vsa_params_t* p, const void* src, void* dst, int inverse, void* hip_stream);

/* Forward (Sec. 2.2; App. B): pooling -> coarse attention -> per-row top-K -> fine
 * block-sparse attention -> gated sum.
 *   q,k,v        in   bf16 [B,H,Np,d] tiled
 *   gate_c       in   bf16 [B,H,Np,d] tiled (G_c)
 *   gate_f       in   bf16 [B,H,Np,d] tiled (G_f), or NULL = ones (Sec. 2.3)
 *   out          out  bf16 [B,H,Np,d] tiled: O_c[cube]*G_c + O_f*G_f, one rounding to bf16
 *                     ([B,Np,H,d] with VSA_FLAG_OUT_TOKEN_MAJOR)
 *   block_idx    out  int32 [B,H,Nc,topk]: selected key cubes of each query cube, ascending
 *                     (the topk largest coarse logits, ties to the lower cube index);
 *                in   when flags has VSA_FLAG_INDICES_GIVEN (must be ascending, distinct,
 *                     each in [0,Nc); not validated: for a list that breaks this the results
 *                     are unspecified, but entries outside [0,Nc) are clamped or skipped, so
 *                     no access leaves the buffers; a query row whose list holds no valid key at
 *                     all -- possible only with such a list, e.g. one made of dead key cubes of 16
 *                     tokens -- gets O_f = 0 and lse_fine = 0)
 *   out_fine     out  bf16 [B,H,Np,d]  O_f           } saved for vsa_backward;
 *   lse_fine     out  fp32 [B,H,Np]    log-sum-exp of the scaled fine logits (0 on pads)
 *   out_coarse   out  fp32 [B,H,Nc,d]  O_c per cube  } any of these four may be NULL
 *   lse_coarse   out  fp32 [B,H,Nc]    log-sum-exp of the coarse logits
 * block_idx may be NULL only without VSA_FLAG_INDICES_GIVEN (the list then lives in the
 * workspace). */
int vsa_forward(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                const void* gate_f, void* out, int32_t* block_idx, void* out_fine, float* lse_fine,
                float* out_coarse, float* lse_coarse, void* workspace, size_t workspace_bytes, void* hip_stream);

/* vsa_forward for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as vsa_forward, minus the workspace: the scratch is a buffer of VSA_STATIC_SCRATCH_MIB MiB
 * that is part of the library itself (one per GPU, held from the library's load until the process
 * ends; vsa_static_scratch_bytes() returns its size).  The call allocates and frees nothing.
 *   - A problem with vsa_workspace_bytes(p, 0) above that size is refused with
 *     VSA_ERR_SCRATCH_LIMIT before anything is enqueued (40 MiB covers the 39936-token, 12-head,
 *     top-78 forward; larger problems go through vsa_forward).
 *   - The first call on a GPU looks the buffer's address up (no allocation); make that call
 *     outside graph capture.
 *   - All calls on one GPU share the buffer.  Every byte a call reads from it was written by
 *     the same call before, so nothing has to be cleared between calls, but two calls that
 *     overlap in time on one GPU (different streams, or graphs replayed side by side) race.
 *   - VSA_FLAG_WORKSPACE_KEPT cannot refer to this buffer: the backward takes a workspace. */
int vsa_forward_static(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                       const void* gate_f, void* out, int32_t* block_idx, void* out_fine, float* lse_fine,
                       float* out_coarse, float* lse_coarse, void* hip_stream);
size_t vsa_static_scratch_bytes(void);

/* Backward of vsa_forward with the selection held constant (Sec. 2.4 states that a
 * backward kernel exists; the gradients are the chain rule through Sec. 2.2's steps:
 * gated sum, fine attention recomputed from lse_fine, coarse attention recomputed from
 * the pooled tensors, mean pooling).  No gradient flows through the top-K.
 *   q,k,v,gate_c,gate_f   as given to vsa_forward
 *   dout         in   bf16 [B,H,Np,d] tiled, gradient of the loss w.r.t. `out` ([B,Np,H,d] with
 *                     VSA_FLAG_OUT_TOKEN_MAJOR)
 *   block_idx, out_fine, lse_fine, out_coarse, lse_coarse   as written by vsa_forward
 *   dq,dk,dv,dgate_c      out  bf16 [B,H,Np,d] tiled
 *   dgate_f      out  bf16 [B,H,Np,d], must be NULL iff gate_f is NULL */
int vsa_backward(const vsa_params_t* p, const void* q, const void* k, const void* v, const void* gate_c,
                 const void* gate_f, const void* dout, const int32_t* block_idx, const void* out_fine,
                 const float* lse_fine, const float* out_coarse, const float* lse_coarse, void* dq, void* dk,
                 void* dv, void* dgate_c, void* dgate_f, void* workspace, size_t workspace_bytes,
                 void* hip_stream);

/* Host-only diagnostic (no GPU, nothing enqueued): replays on the CPU the index arithmetic the
 * kernels apply to a block-index list -- the clamp of the forward and dQ passes, the skip rule and
 * the capacity of the transposed map, the cutting of long transposed lists into runs with numbered
 * partial-result slots -- through the very functions the kernels use, and counts every replayed
 * access that would leave its buffer.  For checking on the CPU that caller-supplied lists of any
 * content (VSA_FLAG_INDICES_GIVEN: entries outside [0,Nc), duplicates, disorder) stay in bounds.
 *   host_block_idx  HOST int32 [B,H,Nc,topk] ([B,H,Nc/4,topk] of tiles with VSA_FLAG_SELECT_POOLED_2X2; entries
 *                   are key cube numbers below 4*Nc with VSA_FLAG_KEY_CUBES_16)
 *   report          HOST int64[8] or NULL: violations, longest transposed list, most dK/dV work
 *                   items and partial-result slots and split lists of a (b,h), most transposed
 *                   entries of a (b,h), split length, slot capacity
 * Returns VSA_OK when no access leaves its buffer, VSA_ERR_BAD_ARG otherwise (or for bad params). */
int vsa_host_replay_lists(const vsa_params_t* p, const int32_t* host_block_idx, int64_t* report);

/* Per-kernel timing for benchmarks (not part of the paper's method).  Between
 * vsa_profile_begin and vsa_profile_end every kernel the other entry points enqueue is
 * bracketed by a pair of HIP events on the caller's stream, up to max_records kernels
 * (events are created inside vsa_profile_begin; further launches are simply not recorded).
 * After the caller has synchronised the stream, record i (launch order) has the static
 * kernel name vsa_profile_name(i) and took vsa_profile_ms(i) milliseconds (-1 on error).
 * One global recorder per process; not thread-safe; host-side calls. */
int vsa_profile_begin(int max_records);
int vsa_profile_count(void);
const char* vsa_profile_name(int i);
float vsa_profile_ms(int i);
int vsa_profile_end(void);

/* Sustained matrix-core rate of the chip, for benchmarks (not part of the paper's method):
 * enqueues ONE kernel that does nothing but v_mfma_f32_32x32x16_bf16 on operands taken from
 * `operands` (DEVICE, 16-byte aligned, at least 65536 bytes of bf16 values; their statistics
 * matter: the clock the chip holds depends on the operand bits), 4 wavefronts per workgroup,
 * `workgroups` workgroups, `iters` x 32 instructions per wavefront, and writes one float per
 * thread to `sink` (DEVICE, workgroups*256 floats).  *flops receives the number of floating
 * point operations of that launch (HOST pointer).  The caller times the launch.
 * Errors: VSA_ERR_NULL, VSA_ERR_BAD_ARG (non-positive counts), VSA_ERR_ALIGN, VSA_ERR_HIP. */
int vsa_bench_mfma_rate(const void* operands, float* sink, int workgroups, int iters, double* flops,
                        void* hip_stream);

/* Human-readable name of a status code (static string, never NULL). */
const char* vsa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* VSA_H_ */
