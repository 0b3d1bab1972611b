/*
 * libfps -- FP8 3D sliding-tile attention (forward) for AMD MI355X (gfx950).
 *
 * C ABI of the hot path of FPSAttention (arXiv 2506.04648): 3D bi-directional attention over the
 * T x H x W token grid of a video latent in which Q, K, V are quantised to FP8 E4M3 with one scale
 * per 3D token tile (Sec. 3.2, Eq. 4-5) and every query tile attends only to the key tiles of a 3D
 * sliding tile window (Sec. 3.1, Eq. 2-3), with the (precision, window) pair optionally chosen per
 * denoising step (Sec. 3.3, Eq. 6; Algorithm 1).
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library allocates no device memory and keeps no state between calls
 *     other than a thread-local error string.
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns without synchronising.
 *   - The return value is an fps_status; on failure fps_last_error() describes it.  Arguments are
 *     validated on the host before anything is launched.  No C++ exception crosses this boundary.
 *   - Every device tensor must be 16-byte aligned.  Inputs are never modified.
 *   - B and heads are interchangeable for the kernels: tensors are indexed by bh = b*heads + h.
 *
 * Token order.  A "raster" tensor is [B, heads, T, H, W, head_dim].  A "tiled" tensor is
 * [B, heads, M*TSP, head_dim]: the grid is zero-padded up to multiples of the tile (Tt,Th,Tw), the
 * tile grid is (nT,nH,nW) = ceil((T,H,W)/(Tt,Th,Tw)), M = nT*nH*nW, TS = Tt*Th*Tw, and token
 * (t,h,w) sits at position u*TSP + r with u = ((t/Tt)*nH + h/Th)*nW + w/Tw and
 * r = ((t%Tt)*Th + h%Th)*Tw + w%Tw (Sec. 3.2 step (1): tokens of one 3D tile are contiguous).
 * TSP = fps_tile_slots(shape) >= TS is the tile's slot count: the kernels work on blocks of 128
 * tokens (32 when that wastes fewer slots, i.e. for TS <= 96), so a tile occupies TS rounded up
 * to whole blocks and shares ONE scale over all of them; the packed operand layouts are per
 * block.  Slots r >= TS, and slots of grid positions outside (T,H,W), are padding: they must be
 * zero in tiled inputs (fps_tile_order writes them so); padded keys never contribute to any
 * output and padded query rows are written as zero.
 *
 * Quantisation sub-tiles (Sec. 3.3 treats the granularity g and the window W as separate
 * hyper-parameters).  With (Qt,Qh,Qw) given, a tile is NS = (Tt/Qt)(Th/Qh)(Tw/Qw) sub-tiles of
 * QS = Qt*Qh*Qw tokens, each rounded up to whole blocks (QSP slots, TSP = NS*QSP) and each with
 * its own scale; in-tile order is then sub-tile-major: token (rt,rh,rw) of the tile sits in slot
 * s*QSP + ((rt%Qt)*Qh + rh%Qh)*Qw + rw%Qw with s = ((rt/Qt)*(Th/Qh) + rh/Qh)*(Tw/Qw) + rw/Qw.
 * Per-tile scale tensors become per-group tensors [B,heads,M*NS], group index u*NS + s
 * (fps_num_groups = M*NS).
 *
 * Supported now: head_dim = 128 and any tile of 1 <= TS <= 32768 tokens, e.g. (1,8,16), (3,4,4),
 * (6,8,8), (12,16,16), (24,32,32), so the granularity g(t) of Sec. 3.2 can change the tile shape
 * from one denoising regime to the next; anything else returns FPS_ERR_UNSUPPORTED.
 */
#ifndef FPS_H
#define FPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FPS_OK = 0,
    FPS_ERR_INVALID_ARG = -1,   /* null pointer, non-positive dimension, misalignment, bad enum */
    FPS_ERR_UNSUPPORTED = -2,   /* valid request outside the implemented shapes                  */
    FPS_ERR_WORKSPACE = -3,     /* reserved                                                      */
    FPS_ERR_HIP = -4            /* a HIP call or kernel launch failed; text in fps_last_error()  */
} fps_status;

typedef enum {
    FPS_PREC_BF16 = 0,   /* no quantisation: bf16 Q,K; fp16 P,V in the PV product; fp32 accumulation */
    FPS_PREC_FP8 = 1     /* Q,K,V,P in E4M3 with per-tile scales (Sec. 3.2)                       */
} fps_precision;

typedef enum {
    FPS_VSCALE_TILE = 0,    /* one V scale per 3D tile, like Q and K                              */
    FPS_VSCALE_CHANNEL = 1  /* one V scale per channel over all tokens (Sec. 3.2, Alg. 1 step 3)  */
} fps_vscale;

typedef enum { FPS_ROLE_Q = 0, FPS_ROLE_K = 1, FPS_ROLE_V = 2 } fps_role;
typedef enum { FPS_OUT_BF16 = 0, FPS_OUT_F32 = 1 } fps_out_dtype;
typedef enum { FPS_LAYOUT_TILED = 0, FPS_LAYOUT_RASTER = 1 } fps_layout;

typedef struct {
    int B, heads, head_dim;   /* head_dim must be 128                                             */
    int T, H, W;              /* real token grid                                                  */
    int Tt, Th, Tw;           /* tile; the padded grid is the grid rounded up to tile multiples   */
    int Qt, Qh, Qw;           /* quantisation sub-tile: 0,0,0 = the tile itself (one scale per
                                 tile); otherwise each must divide Tt, Th, Tw and every sub-tile
                                 has its own scale while the window still counts whole tiles      */
} fps_shape;

typedef enum {
    FPS_EDGE_TRUNCATE = 0,  /* Eq. 2 as a pure distance test: edge tiles see fewer key tiles      */
    FPS_EDGE_SHIFT = 1      /* the window centre is clamped to [r_a, n_a-1-r_a] on each axis, so
                               every query tile sees min(2 r_a + 1, n_a) key tiles per axis       */
} fps_edge;

/* Window in tiles (Eq. 2): with r_a = w_a/2 (integer division), key tile v is kept for query tile
 * u iff |c_a - v_a| <= r_a on each axis a, where c_a = u_a (FPS_EDGE_TRUNCATE: ranges are cut at
 * the grid boundary) or c_a = clamp(u_a, r_a, n_a-1-r_a) (FPS_EDGE_SHIFT; the whole axis if
 * n_a <= 2 r_a + 1).  An even w_a keeps the same tiles as w_a + 1, and w_a >= 2*n_a - 1 keeps the
 * whole axis (dense). */
typedef struct { int wt, wh, ww; fps_edge edge; } fps_window;

/* One regime of the schedule: precision, window W(t), and the granularity g(t) (Eq. 6) as a tile
 * and, optionally, a quantisation sub-tile.  Tt = Th = Tw = 0 means "whatever tile the shape of
 * the call has", Qt = Qh = Qw = 0 "whatever sub-tile it has". */
typedef struct { fps_precision prec; fps_window win; int Tt, Th, Tw; int Qt, Qh, Qw; } fps_regime;

/* Denoising-step-aware schedule (Eq. 6): step t in 1..num_steps, thresholds t1 = alpha1*num_steps,
 * t2 = alpha2*num_steps evaluated in float; regime[0] if t <= t1, regime[1] if t1 < t <= t2,
 * regime[2] otherwise.  Requires 0 < alpha1 < alpha2 < 1. */
typedef struct {
    int step, num_steps;
    float alpha1, alpha2;
    fps_regime regime[3];
} fps_step_cfg;

/* Thread-local description of the last failure on the calling thread; never NULL. */
const char* fps_last_error(void);

/* ---- host-only helpers (no device work) ------------------------------------------------- */

/* Eq. 6 / Algorithm 1 step 1.  Writes the selected regime to *out. */
int fps_schedule_select(const fps_step_cfg* cfg, fps_regime* out);

/* M, the number of tiles per head, or 0 on an invalid shape. */
size_t fps_num_tiles(const fps_shape* shape);

/* M*NS, the number of quantisation groups (scales) per head, or 0 on an invalid shape. */
size_t fps_num_groups(const fps_shape* shape);

/* TSP, the slots one tile occupies in tiled and packed tensors (TS rounded up to whole blocks),
 * or 0 on an invalid shape. */
size_t fps_tile_slots(const fps_shape* shape);

/* BS, the slots of one block (the unit the kernels stage and a workgroup's query rows): 128, or 32
 * when a quantisation group has at most 96 tokens; TSP is a multiple of it.  0 on an invalid shape. */
size_t fps_block_slots(const fps_shape* shape);

/* Bytes of one packed tensor for the given precision (all B*heads): M*TSP*head_dim bytes for FP8,
 * twice that for BF16.  0 on an invalid shape. */
size_t fps_packed_bytes(const fps_shape* shape, fps_precision prec);

/* Host statement of the tile neighbourhood of Eq. 2: mask[u*M + v] = 1 iff key tile v is kept for
 * query tile u.  `mask` is host memory of M*M bytes.  Also returns the number of kept pairs
 * through *pairs_or_null (the M x |W(u)| dense blocks of Sec. 3.1). */
int fps_tile_mask_host(const fps_shape* shape, const fps_window* win, uint8_t* mask,
                       uint64_t* pairs_or_null);

/* ---- device entry points ------------------------------------------------------------------ */

/* Sec. 3.2 step (1).  raster bf16 [B,heads,T,H,W,128] (device) -> tiled bf16 [B,heads,M*TSP,128]
 * (device), padded slots written as zero. */
int fps_tile_order(const fps_shape* shape, const void* x_raster_bf16, void* x_tiled_bf16,
                   void* stream);

/* Inverse of fps_tile_order for outputs: tiled [B,heads,M*TSP,128] of dtype `dt` (device) ->
 * raster [B,heads,T,H,W,128] of the same dtype (device). */
int fps_tile_unorder(const fps_shape* shape, const void* o_tiled, fps_out_dtype dt, void* o_raster,
                     void* stream);

/* Eq. 4-5 (Algorithm 1 steps 2-3).  Tiled bf16 (device) -> E4M3 codes in the library's packed
 * operand layout for `role` (device, fps_packed_bytes(shape, FPS_PREC_FP8) bytes) and fp32 scales
 * (device): [B,heads,M*NS] for per-group scales (one per tile, or per quantisation sub-tile),
 * [B,heads,128] for FPS_VSCALE_CHANNEL (role V only).
 * scale = amax/448 as a correctly rounded float division (1.0 for an all-zero group); code =
 * round-to-nearest-even, saturating, of the exact quotient x/scale.  `vscale` is ignored for
 * roles Q and K. */
int fps_quantize_tiles(const fps_shape* shape, const void* x_tiled_bf16, fps_role role,
                       fps_vscale vscale, void* xq_out, float* scales_out, void* stream);

/* fps_tile_order fused into fps_quantize_tiles (Sec. 3.2 steps (1)+(2) in one pass over HBM): the
 * input is the RASTER bf16 tensor [B,heads,T,H,W,128] (device); each workgroup gathers the tokens
 * of its 3D tile (padded slots read as zero) and proceeds exactly like fps_quantize_tiles.
 * Outputs, scales and codes are bit-identical to fps_tile_order followed by fps_quantize_tiles. */
int fps_quantize_raster(const fps_shape* shape, const void* x_raster_bf16, fps_role role,
                        fps_vscale vscale, void* xq_out, float* scales_out, void* stream);

/* BF16-mode counterpart of fps_quantize_tiles: re-lays a tiled bf16 tensor (device) into the
 * packed operand layout for `role` (device, fps_packed_bytes(shape, FPS_PREC_BF16) bytes).
 * Q and K keep their bf16 values.  V is stored as fp16 after an exact per-tile power-of-two
 * scaling (so that P can be held in fp16, 11 significant bits, in the PV product); the scales
 * 2^e go to vscale_out, fp32 [B,heads,M*NS] (device), required for role V and ignored otherwise.
 * bf16 values more than 2^28 times smaller than their tile's largest magnitude lose precision. */
int fps_pack_tiles_bf16(const fps_shape* shape, const void* x_tiled_bf16, fps_role role,
                        void* xp_out, float* vscale_out, void* stream);

/* fps_tile_order fused into fps_pack_tiles_bf16: the input is the RASTER bf16 tensor
 * [B,heads,T,H,W,128] (device).  Outputs are bit-identical to fps_tile_order followed by
 * fps_pack_tiles_bf16. */
int fps_pack_raster_bf16(const fps_shape* shape, const void* x_raster_bf16, fps_role role,
                         void* xp_out, float* vscale_out, void* stream);

/* Debug: packed E4M3 tensor (device) -> plain row-major codes [B,heads,M*TSP,128] (device). */
int fps_debug_unpack_q8(const fps_shape* shape, const void* xq, fps_role role,
                        uint8_t* codes_rowmajor, void* stream);

/* Debug: plain device-to-device copy of `bytes` bytes (a positive multiple of 16; src and dst are
 * device memory and must not overlap).  A kernel of exactly known HBM traffic, used to calibrate
 * the profiler's FETCH_SIZE / WRITE_SIZE counters. */
int fps_debug_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Debug: a kernel that does nothing but issue the FP8 matrix instruction of the attention kernel
 * (v_mfma_f32_16x16x128_f8f6f4, 8 independent accumulator chains per wave, no memory traffic in
 * the loop): `workgroups` workgroups of 256 threads, `iters` loop trips of 8 instructions per
 * wave.  FLOPs launched = workgroups * 4 waves * iters * 8 * 65536.  Timed by the caller, it gives
 * the matrix rate the chip sustains, the yardstick next to the datasheet peak.  `sink` is device
 * memory of workgroups*256 floats that receives one value per thread. */
int fps_debug_mfma_rate(int workgroups, int iters, float* sink, void* stream);

/* Debug: how matrix and vector instructions share a SIMD's issue port -- the bound of the attention
 * kernels, whose softmax puts a dozen vector instructions beside every matrix instruction
 * (Sec. 3.4 calls the kernel tensor-core bound; this measures what the chip allows).  The kernel
 * loops `iters` times over 8 groups, a group being one matrix instruction (matrix_kind 0:
 * v_mfma_f32_16x16x128_f8f6f4 on E4M3; 1: v_mfma_f32_16x16x32_bf16; 2: none;
 * 3: v_mfma_f32_32x32x64_f8f6f4 on E4M3, twice the work of 0; 4: v_mfma_f32_32x32x16_bf16, twice
 * the work of 1) followed by
 * valu_per_mfma (one of 0 1 2 3 4 6 8 12 16 24 32) vector units (valu_kind 0: one v_fma_f32; 1: one
 * v_exp_f32 plus one v_add_f32), with no memory traffic.  `workgroups` workgroups of 256 threads
 * are launched, each reserving 1/workgroups_per_cu of a compute unit's LDS so that exactly that
 * many share a SIMD per wave slot.  cycles (device, workgroups*4 entries) receives each wave's
 * shader-clock count for the whole loop; sink (device, workgroups*256 floats) one value per
 * thread. */
int fps_debug_issue_mix(int matrix_kind, int valu_per_mfma, int valu_kind, int workgroups_per_cu,
                        int workgroups, int iters, float* sink, unsigned long long* cycles,
                        void* stream);

/* Debug: the raw score accumulators sum_c qcode_ic * kcode_jc (before the s^Q s^K / sqrt(d)
 * dequantisation of Eq. 3) of query tile u and key tile v of head bh, computed with the same
 * matrix instruction as fps_attn_fwd; `scores` is device memory of TSP*TSP floats, [query][key]
 * in in-tile slot order (entries of padding slots are zero products).  Used to measure the
 * accumulation accuracy of the hardware; refused for TSP > 4096. */
int fps_debug_scores_q8(const fps_shape* shape, const void* q, const void* k, int bh, int u, int v,
                        float* scores, void* stream);

/* Debug: the same accumulators for ONE block pair, for tiles too large for the call above: query
 * block jq of tile u against key block jk of tile v (blocks of BS = 32 or 128 slots, BS = TSP /
 * blocks per tile; jq, jk in 0 .. TSP/BS - 1); `scores` is device memory of BS*BS floats,
 * [query][key] in slot order within the blocks.  *bs_or_null receives BS (host memory). */
int fps_debug_scores_block_q8(const fps_shape* shape, const void* q, const void* k, int bh, int u,
                              int jq, int v, int jk, float* scores, int* bs_or_null, void* stream);

/* Eq. 2-3 and Sec. 3.2 "aggregation and dequantisation" (Algorithm 1 steps 4-5).
 *   q, k, v    packed tensors (device) made by fps_quantize_tiles (FP8) or fps_pack_tiles_bf16
 *              (BF16) with roles Q, K, V for the same shape.
 *   sq, sk, sv fp32 scales (device) from fps_quantize_tiles; in BF16 mode sq and sk are ignored
 *              (may be NULL) and sv is the vscale_out of fps_pack_tiles_bf16.
 *   step       if non-NULL, (prec, win) are replaced by fps_schedule_select(step); the packed
 *              tensors must match the selected precision, and if the selected regime names a
 *              tile or a sub-tile it must be that of `shape` (the inputs were quantised with
 *              it), else FPS_ERR_INVALID_ARG.
 *   out        of dtype out_dt (device): tiled [B,heads,M*TSP,128] with padded query rows set to 0
 *              (FPS_LAYOUT_TILED), or raster [B,heads,T,H,W,128] holding the real tokens only
 *              (FPS_LAYOUT_RASTER: the inverse tile ordering is fused into the epilogue).
 *   visited    NULL, or device memory of M*M bytes zeroed by the caller: the kernel sets
 *              visited[u*M+v] = 1 for every tile pair it computes (written by head 0 only).
 * Scores are dequantised per pair of quantisation groups (s^Q * s^K / sqrt(d); per tile pair
 * without sub-tiles); softmax runs online in base 2
 * with an integer row reference; P is rounded to E4M3 after scaling by 448 (FP8) or to fp16
 * (BF16); the denominator sums the unrounded P. */
int fps_attn_fwd(const fps_shape* shape, const fps_window* win, fps_precision prec,
                 const fps_step_cfg* step, const void* q, const void* k, const void* v,
                 const float* sq, const float* sk, const float* sv, fps_vscale vscale, void* out,
                 fps_out_dtype out_dt, fps_layout out_layout, uint8_t* visited, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FPS_H */
