/*
 * distgrid.h -- C ABI of the MI355X (gfx950) library for the DistGrid training hot path
 * (DistGrid: Scalable Scene Reconstruction with Distributed Multi-resolution Hash Grid,
 *  arXiv 2405.04416).
 *
 * Conventions, valid for every entry point unless its comment says otherwise:
 *  - every function returns int: DG_OK, or a negative DG_ERR_* code; argument checks run
 *    synchronously on the host before anything is enqueued; dg_last_error() returns a
 *    human-readable description of the last failure on the calling thread;
 *  - "device" pointers are HIP device memory owned by the caller; the library never
 *    allocates, frees or retains them; "host" pointers are ordinary memory;
 *  - all work is enqueued on the caller's stream (a hipStream_t passed as void*; NULL is
 *    the default stream) and the call returns without synchronising;
 *  - arrays are row-major, innermost dimension last; fp16 means IEEE binary16;
 *  - outputs documented as "+=" accumulate into what the buffer holds (the caller zeroes
 *    it); all other outputs are overwritten;
 *  - data-dependent overflow (more than k_max segments on a ray, more samples than the
 *    caller's capacity) is reported through a device-side status word, not through the
 *    return code.
 */
#ifndef DISTGRID_H
#define DISTGRID_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DG_OK               0
#define DG_ERR_ARG         (-1)  /* null / misaligned / inconsistent argument          */
#define DG_ERR_UNSUPPORTED (-2)  /* a shape the kernels are not built for              */
#define DG_ERR_WORKSPACE   (-3)  /* workspace smaller than the *_workspace_bytes query */
#define DG_ERR_HIP         (-4)  /* a HIP call or kernel launch failed                 */

#define DG_F32 0u
#define DG_F16 1u
#define DG_MAX_LEVELS 16
#define DG_MAX_PARTITIONS 64

const char *dg_last_error(void);

/* ------------------------------------------------------------------------------------
 * Deformable multi-resolution hash grid (Sec. 3.2, Sec. 4.1).
 * A host-side descriptor, built once per sub-model and passed by pointer (it is copied).
 * Level l has n_voxels[l] = floor(N_min * growth^l) voxels along the longest box axis
 * (Instant-NGP Eq. 2-3), res[l][d] = ceil(a_d/s * n_voxels[l]) voxels along axis d
 * (Sec. 4.1), cubic voxels of side s/n_voxels[l].  A level whose vertex count
 * prod(res+1) is <= T = 2^log2_T is stored one-to-one (x fastest), otherwise its
 * vertices are hashed into T entries (Sec. 4.1; hash: Instant-NGP Eq. 4).  Level l
 * occupies entries [offset[l], offset[l+1]) of the table, each entry n_features floats.
 * A sample with unit coordinates u in [0,1]^3 (clamped) sits at grid position
 * u_d * scale[l][d] (one fp32 multiply), in the cell floor(.) clamped to res-1.
 * ---------------------------------------------------------------------------------- */
typedef struct dg_grid_desc {
    uint32_t n_levels;                    /* L <= 16                      */
    uint32_t n_features;                  /* F, must be 2                 */
    uint32_t log2_T;
    uint32_t n_entries;                   /* offset[n_levels]             */
    uint32_t n_voxels[DG_MAX_LEVELS];
    uint32_t res[DG_MAX_LEVELS][3];
    uint32_t dense[DG_MAX_LEVELS];
    uint32_t offset[DG_MAX_LEVELS + 1];
    float    scale[DG_MAX_LEVELS][3];
} dg_grid_desc;

/* growth factor b = exp((ln N_max - ln N_min) / (L-1)) (Instant-NGP Eq. 3). */
double dg_growth_factor(uint32_t N_min, uint32_t N_max, uint32_t L);
/* Fills *desc (host).  extent = side lengths (a,b,c) of the sub-model's box.
 * DG_ERR_ARG on null pointers or non-positive extents, DG_ERR_UNSUPPORTED if L > 16,
 * F != 2, log2_T > 24 or the table would exceed 2^32 entries. */
int dg_grid_desc_init(dg_grid_desc *desc, uint32_t L, uint32_t F, uint32_t log2_T,
                      uint32_t N_min, double growth, const double extent[3]);

/* ------------------------------------------------------------------------------------
 * Ray / box segments and their distribution to partitions (Sec. 4.2.1, Sec. 4.4.2,
 * Fig. 2 steps 2-3).
 * o, d [R,3] fp32 device; parts [P,6] fp32 device, each (lo_x,lo_y,lo_z,hi_x,hi_y,hi_z),
 * closely paved and non-overlapping, neighbours storing the same float for a shared face.
 * Slab test in fp32 with one rounding per operation: t = (face - o) * (1/d); a ray
 * parallel to a slab is inside iff lo <= o < hi.  A box is hit iff t_out > max(t_near,
 * t_min).  Per ray the hits are ordered front to back (ties by box index); the first
 * k_max are kept and bit 0 of *status is set if any ray had more.
 * Outputs (device): seg_count [R]; seg_t [R,k_max,2] = (t_in,t_out), consecutive segments
 * share a bit-identical boundary; seg_part [R,k_max] box index (-1 in unused slots).
 * If part_offset is non-null the (ray,slot) pairs are also distributed to their boxes by
 * a stable counting sort: part_offset [P+1], seg_ray / seg_slot [R*k_max capacity] hold
 * box p's segments at [part_offset[p], part_offset[p+1]) in ascending (ray,slot) order.
 * That step needs dg_segments_workspace_bytes(R,P) bytes of device workspace.
 * holes: NULL, or [P,6] fp32 device boxes: partition p then covers parts[p] minus holes[p]
 * (Sec. 4.2.2: the coarse sub-models of the two-level cascade cover the outer box around the
 * inner one, split by the same planes).  The hole's interval on the ray comes from the same
 * slab expressions; the region is met in up to two pieces, [t_in, min(hole entry, t_out)] and
 * [max(hole exit, t_in), t_out] (a hole may overhang its box, e.g. the whole inner box given as
 * the hole of every outer partition), each kept if it has positive length and listed under box index p.  A hole with no
 * volume (hi <= lo on some axis) is no hole.  Faces that a hole shares with another box give
 * bit-identical times, so fine and coarse pieces pave the ray as plain boxes do.
 * P <= DG_MAX_PARTITIONS, 1 <= k_max <= 12.
 * ---------------------------------------------------------------------------------- */
size_t dg_segments_workspace_bytes(uint32_t R, uint32_t P);
int dg_ray_aabb_segments(const float *o, const float *d, uint32_t R,
                         const float *parts, const float *holes, uint32_t P, float t_min, uint32_t k_max,
                         uint32_t *seg_count, float *seg_t, int32_t *seg_part,
                         uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot,
                         uint32_t *status, void *ws, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): dg_ray_aabb_segments with the counter table of the distribution step in a fixed device array of the
 * library (1 MiB per GPU the library runs on, held until the process ends) instead of a workspace.  Same arguments
 * without ws / ws_bytes, same results.  Limit: ceil(R/256) * P <= DG_SEGMENTS_STATIC_COUNTERS = 2^18 counters (2^20
 * rays with 64 boxes, 2^24 rays with 4); beyond that DG_ERR_WORKSPACE and nothing is enqueued.  The call allocates and
 * frees nothing; the first call on a device looks the array's address up (hipGetSymbolAddress) with that device
 * current.  Every call on a GPU uses that GPU's one array (each call rewrites all counters it reads, so nothing is
 * cleared in between): calls that overlap on one GPU -- two streams, two threads -- race; serialise them. */
#define DG_SEGMENTS_STATIC_COUNTERS (1u << 18)
int dg_ray_aabb_segments_static(const float *o, const float *d, uint32_t R,
                                const float *parts, const float *holes, uint32_t P, float t_min, uint32_t k_max,
                                uint32_t *seg_count, float *seg_t, int32_t *seg_part,
                                uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot,
                                uint32_t *status, void *stream);

/* Stratified jittered samples of the n_seg segments listed in seg_ray/seg_slot (device,
 * already offset to one box's list), all inside box `box` (host, 6 floats).
 * Sample s of a segment: dt = (t_out-t_in)/S, t = t_in + (s+xi)*dt, x = fma(t,d,o),
 * u = (x-lo) * (1/(hi-lo)); each step one fp32 rounding.  xi in [0,1) is jitter[j*S+s]
 * if jitter != NULL, else a counter-based generator keyed by (seed, ray, slot, s):
 * splitmix64 output mix of seed + 0x9E3779B97F4A7C15*(ctr+1), ctr = ray<<32|slot<<16|s,
 * top 24 bits scaled by 2^-24.
 * Outputs (device): u [n_seg*S,3] fp32 unit coordinates, delta [n_seg*S] stratum widths,
 * t [n_seg*S] the sample distances along the ray (NULL: not wanted; the depth channel needs them). */
int dg_sample_segments(const float *o, const float *d, const float *seg_t,
                       const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t n_seg,
                       uint32_t k_max, const float *box, uint32_t S, uint64_t seed,
                       const float *jitter, float *u, float *delta, float *t, void *stream);

/* Direction encoding: real spherical harmonics of bands 0..degree-1 (degree 1..4) of the
 * normalised direction of ray index[i] (index NULL: i itself); out [n, degree^2] fp16.
 * Band l, order m is stored at l*l + l + m; Condon-Shortley phase included. */
int dg_dir_encode(const float *d, const uint32_t *index, uint64_t n, uint32_t degree,
                  void *out, void *stream);

/* ------------------------------------------------------------------------------------
 * Hash-grid encode (Sec. 3.2): feature f of level l of sample n = sum over the 8 cell
 * corners of w_c * table[entry_c, f], trilinear weights w_c, entry by dense map or hash.
 * table [n_entries, F] fp32 device; u [N,3] fp32 device.
 * Feature layout, here and in every call below that takes features or their gradient:
 * LEVEL-MAJOR planes, feat [L, N, F] (the concatenated embedding of sample n is the
 * column feat[:, n, :]); fp32 or fp16 (feat_dtype DG_F32 / DG_F16; fp16 is rounded once
 * from the fp32 sum).  Kernels walk one level at a time, so planes keep their accesses
 * contiguous.
 * ---------------------------------------------------------------------------------- */
int dg_hashgrid_encode_fwd(const dg_grid_desc *desc, const float *table, const float *u,
                           uint64_t N, void *feat, uint32_t feat_dtype, void *stream);
/* Transpose of the above: dtable[entry_c, f] += w_c * dfeat[l, n, f]; the summation order is not
 * fixed.  dfeat [L, N, F] fp32 device (level-major planes); dtable "+=".
 * With ws == NULL every contribution is a global fp32 atomic (after merging lanes that share a cell).
 * With a workspace of dg_hashgrid_encode_bwd_workspace_bytes(desc, N) bytes the contributions are
 * binned by table region and summed in on-chip memory first (much faster for large N); on that path a
 * contribution is rounded to 18 mantissa bits (relative error at most 2^-20, unbiased) before it is
 * summed exactly (in fixed point scaled to the batch's largest magnitude: a contribution below 2^-32 of that magnitude
 * adds nothing).  If any contribution of the batch is infinite or NaN the sums cannot be formed: every table region
 * that received contributions then gets NaN in its first entry, so the gradient is visibly non-finite as it would be
 * with fp32 atomics.  ws must be 256-byte aligned; a smaller workspace is accepted and makes the call run
 * in batches, DG_ERR_WORKSPACE if it cannot hold one tile of 512 samples (16 bytes per sample, level
 * and pair of corners, plus bookkeeping). */
size_t dg_hashgrid_encode_bwd_workspace_bytes(const dg_grid_desc *desc, uint64_t N);
int dg_hashgrid_encode_bwd(const dg_grid_desc *desc, const float *u, const float *dfeat,
                           uint64_t N, float *dtable, void *ws, size_t ws_bytes, void *stream);
/* The binned pass in two parts, for callers that want the first part out of the way early: the sizes of the bin queues
 * depend on the coordinates alone, so they can be counted as soon as u exists -- on another stream, beside the forward
 * pass -- and the backward pass then starts with the queues laid out.
 * dg_hashgrid_encode_bwd_count: the count sweep and its scans for all N samples; ws must hold them in one batch
 * (dg_hashgrid_encode_bwd_workspace_bytes(desc, N) bytes), else DG_ERR_WORKSPACE.
 * dg_hashgrid_encode_bwd_counted: dg_hashgrid_encode_bwd without that part.  The counts must come from a
 * dg_hashgrid_encode_bwd_count call with the same desc, u, N, ws and ws_bytes that has completed before this call's work
 * starts (same stream, or an event between the streams), and nothing else may have used ws in between; the results are
 * those of dg_hashgrid_encode_bwd. */
int dg_hashgrid_encode_bwd_count(const dg_grid_desc *desc, const float *u, uint64_t N, void *ws, size_t ws_bytes,
                                 void *stream);
int dg_hashgrid_encode_bwd_counted(const dg_grid_desc *desc, const float *u, const float *dfeat,
                                   uint64_t N, float *dtable, void *ws, size_t ws_bytes, void *stream);
/* Absolute table entry of every corner: idx [N, L, 8] uint32, corner c = cx + 2cy + 4cz. */
int dg_hashgrid_corner_indices(const dg_grid_desc *desc, const float *u, uint64_t N,
                               uint32_t *idx, void *stream);

/* ------------------------------------------------------------------------------------
 * Field MLPs (Sec. 3.2: a small MLP fuses the level features; Sec. 5.1: sigmoid hidden activation in the colour
 * net, outputs of both nets clipped to [-15,15] before the output activations).
 *   density: feat[n_feat] -> n_hidden_d (ReLU) -> geo[n_geo];  sigma = exp(clip(geo[0]))
 *   colour : [geo | dir_enc] -> n_hidden_c (act_c) [-> n_hidden_c (act_c)] -> 3;
 *            rgb = sigmoid(clip(.))
 * No biases.  Inputs, weights and every hidden activation are fp16 (round to nearest
 * even), products accumulate in fp32.  weights: fp16 device, the matrices
 * Wd1[n_hidden_d,n_feat], Wd2[n_geo,n_hidden_d], Wc1[n_hidden_c,n_geo+n_dir],
 * (Wc2[n_hidden_c,n_hidden_c]), Wc3[3,n_hidden_c] one after another, each [out,in].
 * feat [n_feat/2, N, 2] fp16 (the encode's level-major planes; input i of sample n is
 * feat[i/2, n, i%2]); dir_enc [ceil(N/S), n_dir] fp16, row n/S serves sample n.
 * Outputs: sigma [N] fp32, rgb [N,3] fp32.
 * Supported shapes: (n_feat,n_hidden_d,n_geo,n_dir,n_hidden_c,n_layers_c) =
 * (32,64,16,16,64,2) and (8,32,16,4,32,1); others return DG_ERR_UNSUPPORTED.
 * ---------------------------------------------------------------------------------- */
typedef struct dg_mlp_desc {
    uint32_t n_feat, n_hidden_d, n_geo, n_dir, n_hidden_c, n_layers_c;
    uint32_t act_c;                       /* 0 ReLU, 1 sigmoid */
    uint32_t n_app;                       /* appearance inputs of the colour net: 0, 16 or 48 (Sec. 4.4.3) */
} dg_mlp_desc;
size_t dg_mlp_weight_count(const dg_mlp_desc *desc);
int dg_mlp_fwd(const dg_mlp_desc *desc, const void *weights, const void *feat,
               const void *dir_enc, uint32_t S, uint64_t N, float *sigma, float *rgb,
               void *stream);
/* Backward of the above; activations are recomputed, nothing is saved by dg_mlp_fwd.
 * dsigma [N], drgb [N,3] fp32.  Every back-propagated delta is multiplied by loss_scale
 * (a power of two is advisable) before it is rounded to fp16, and dfeat / dW are divided
 * by it again in fp32.  Outputs: dfeat [n_feat/2, N, 2] fp32 planes (overwritten); dW fp32, "+=",
 * same packing as weights.  ws: dg_mlp_bwd_workspace_bytes(desc, N) bytes, 256-byte aligned. */
size_t dg_mlp_bwd_workspace_bytes(const dg_mlp_desc *desc, uint64_t N);
int dg_mlp_bwd(const dg_mlp_desc *desc, const void *weights, const void *feat,
               const void *dir_enc, uint32_t S, uint64_t N, const float *dsigma,
               const float *drgb, float loss_scale, float *dfeat, float *dW,
               void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------
 * Local volume rendering of one box's segments (Eq. 3 by quadrature; Fig. 2 step 4):
 * alpha_i = 1-exp(-sigma_i delta_i), T_i = prod_{j<i}(1-alpha_j),
 * C_k = sum_i T_i alpha_i c_i, T_k = prod_i (1-alpha_i).
 * sigma, delta [n_seg*S], rgb [n_seg*S,3] fp32 device; segment j belongs to ray
 * seg_ray[j], slot seg_slot[j]; results are written to Ck [R,k_max,3], Tk [R,k_max]
 * at that (ray,slot) (Fig. 2 step 5).
 * ---------------------------------------------------------------------------------- */
int dg_composite_segment_fwd(const float *sigma, const float *rgb, const float *delta,
                             uint32_t n_seg, uint32_t S, const uint32_t *seg_ray,
                             const uint32_t *seg_slot, uint32_t k_max, float *Ck, float *Tk,
                             void *stream);
/* Depth for evaluation rendering (Sec. 4.4.2: the sub-models' partial results are merged into colour, depth and
 * transmittance of the ray): D_k = sum_i T_i alpha_i t_i with the weights above, t [n_seg*S] the sample distances from
 * dg_sample_segments; written to Dk [R,k_max] at the segment's (ray, slot). */
int dg_composite_segment_depth(const float *sigma, const float *delta, const float *t, uint32_t n_seg, uint32_t S,
                               const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max, float *Dk,
                               void *stream);
/* Backward: from gCk [R,k_max,3], gTk [R,k_max] to dsigma [n_seg*S], drgb [n_seg*S,3]. */
int dg_composite_segment_bwd(const float *sigma, const float *rgb, const float *delta,
                             uint32_t n_seg, uint32_t S, const uint32_t *seg_ray,
                             const uint32_t *seg_slot, uint32_t k_max, const float *gCk,
                             const float *gTk, float *dsigma, float *drgb, void *stream);

/* Segmented volume rendering (Eq. 5, 6; Fig. 2 step 6): C = sum_k (prod_{j<k} T_j) C_k,
 * T = prod_k T_k over the first seg_count[r] slots; a ray with no segment gives C=0, T=1. */
int dg_merge_segments(const float *Ck, const float *Tk, const uint32_t *seg_count,
                      uint32_t R, uint32_t k_max, float *C, float *T, void *stream);
/* Depth merges like a colour channel under Eq. 5: D = sum_k (prod_{j<k} T_j) D_k; D [R] (0 for a ray with no
 * segment). */
int dg_merge_depth(const float *Dk, const float *Tk, const uint32_t *seg_count, uint32_t R, uint32_t k_max,
                   float *D, void *stream);
/* Its backward (Eq. 7, 8), evaluated without dividing by any T_k; unused slots get 0. */
int dg_merge_segments_bwd(const float *Ck, const float *Tk, const uint32_t *seg_count,
                          uint32_t R, uint32_t k_max, const float *gC, const float *gT,
                          float *gCk, float *gTk, void *stream);

/* Loss seeds (Eq. 9 as a mean over rays, Eq. 10 weighted by lambda1):
 * gC = 2 (C - Cgt)/R, gT = lambda1 / (R (1-T)) where 1-T >= 1e-6, else 0;
 * *loss (device scalar, "+=", may be NULL) accumulates the loss value. */
int dg_loss_seed(const float *C, const float *T, const float *Cgt, uint32_t R,
                 float lambda1, float *gC, float *gT, float *loss, void *stream);

/* The same networks with appearance features (Sec. 4.4.3: a fixed vector per image, 16 or 48 values, as additional
 * inputs of the colour net): colour input = [geo | dir_enc row | app row], desc->n_app = 16 or 48 (0: app is ignored and
 * may be NULL; only the 32-64-16 / 64-64-3 shape takes appearance inputs).  app [ceil(N/S), n_app] fp16 device, 16-byte
 * aligned, row n/S serves sample n like dir_enc.  Weight packing: the five matrices as above, Wc1 [n_hidden_c, n_geo+n_dir]
 * included, then Wapp [n_hidden_c, n_app] -- the columns of the first colour layer that multiply the appearance
 * features, kept last so that the packing of the other matrices does not depend on n_app; dW likewise.  The appearance
 * features get no gradient (they are fixed).  Workspace: dg_mlp_bwd_app_workspace_bytes(desc, N, S) bytes (it holds
 * 256 bytes per ROW of samples on top of what dg_mlp_bwd needs). */
int dg_mlp_fwd_app(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                   const void *app, uint32_t S, uint64_t N, float *sigma, float *rgb, void *stream);
size_t dg_mlp_bwd_app_workspace_bytes(const dg_mlp_desc *desc, uint64_t N, uint32_t S);
int dg_mlp_bwd_app(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                   const void *app, uint32_t S, uint64_t N, const float *dsigma, const float *drgb,
                   float loss_scale, float *dfeat, float *dW, void *ws, size_t ws_bytes, void *stream);
/* Row table for the two calls above: out[i, :] = table[image_of_ray[index[i]], :] (index NULL: i itself);
 * table [n_images, n_app] fp16, image_of_ray [R] uint32, out [n, n_app] fp16; n_app a multiple of 8. */
int dg_appearance_rows(const void *table, const uint32_t *image_of_ray, const uint32_t *index, uint64_t n,
                       uint32_t n_app, void *out, void *stream);

/* Evaluation rendering (Sec. 4.4.2: every sub-model renders its segments, the partial colour, depth and transmittance are
 * merged into the final result), forward only and fused: dg_mlp_fwd_app, dg_composite_segment_fwd and
 * dg_composite_segment_depth on the n_seg segments of S samples each in one kernel, so that the densities and colours of
 * the samples are never written to memory.  Inputs as for dg_mlp_fwd_app with N = n_seg * S (feat [n_feat/2, N, 2] fp16,
 * dir_enc / app one row per segment), delta and t [N] from dg_sample_segments; outputs Ck [R,k_max,3], Tk [R,k_max] and
 * Dk [R,k_max] at each segment's (ray, slot).  t == NULL and Dk == NULL together: no depth.  Same arithmetic as the three
 * separate calls.  DG_ERR_UNSUPPORTED unless the network is the 32-64-16 / (32 + n_app)-64-64-3 one and S <= 64 (one
 * wavefront renders a segment); callers then use the separate entry points. */
int dg_mlp_composite_fwd(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                         const void *app, uint32_t S, uint32_t n_seg, const float *delta, const float *t,
                         const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max, float *Ck, float *Tk,
                         float *Dk, void *stream);

/* One Adam step (Sec. 5.1 names the optimiser; the update is Algorithm 1 of Kingma & Ba) on n fp32 values, in place:
 *   g' = g + l2 * p;  m = beta1 m + (1 - beta1) g';  v = beta2 v + (1 - beta2) g'^2;
 *   p -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps),      step = 1, 2, ...
 * param, grad, m, v: device arrays of n floats, 16-byte aligned, owned by the caller.  grad is consumed: every
 * gradient that was used is set to 0, so the next backward pass can accumulate without a separate clearing pass.
 * skip_zero_grad != 0 (for the hash tables): a value whose gradient is exactly 0 is left alone altogether -- value
 * and both moments unchanged -- and the sweep does not fetch them (the rule of the system whose unnamed
 * hyper-parameters Sec. 5.1 inherits: beta1 0.9, beta2 0.99, eps 1e-15, l2 1e-6 on the MLP weights only).
 * param_half: NULL, or a device array of n fp16 values (8-byte aligned) that receives the rounded new values of
 * every value that was updated (the MLP kernels read fp16 weights).  Errors: DG_ERR_ARG for null / misaligned
 * pointers, step == 0, beta outside [0, 1), eps < 0; DG_ERR_UNSUPPORTED for n >= 2^41. */
int dg_adam_step(float *param, float *grad, float *m, float *v, uint64_t n, float lr, float beta1, float beta2,
                 float eps, uint32_t step, float l2, uint32_t skip_zero_grad, void *param_half, void *stream);

/* Learning rate of Sec. 5.1 (host function): lr0 at iteration 0 down to lr1 at `total` along half a cosine,
 * lr1 afterwards (the paper: 0.05 -> 0.005 over 300 000 iterations). */
float dg_cosine_lr(float lr0, float lr1, uint64_t iteration, uint64_t total);

/* ------------------------------------------------------------------------------------
 * Occupancy grid and occupancy-guided sampling (Sec. 3.2: per-voxel densities let ray
 * marching skip empty space; Sec. 4.1: the grid is deformable like the hash grid; Sec. 5.1:
 * one scale, plain x-fastest storage, resolution 512, decay 0.99 every 16 iterations,
 * warm-up of 4096 iterations, bit threshold 0.6 before iteration 10 000 and 60 after; the
 * refresh rule -- decay, candidate cells, maximum, threshold -- is Instant-NGP App. E.2).
 * The grid has res[d] = ceil(a_d/s * N) cubic cells of side s/N; a point with unit
 * coordinates u (clamped to [0,1]) lies in cell min(floor(u_d * scale[d]), res[d]-1) per
 * axis, linear index x + res_x (y + res_y z).  density: n_cells fp32 (device);
 * bits: ceil(n_cells/32) uint32 words (device), bit c%32 of word c/32 belongs to cell c.
 * ---------------------------------------------------------------------------------- */
typedef struct dg_occ_desc {
    uint32_t res[3];
    uint32_t n_cells;
    float    scale[3];
} dg_occ_desc;
/* Host.  DG_ERR_ARG for null pointers, N == 0 or non-positive extents, DG_ERR_UNSUPPORTED for more than 2^31 cells. */
int dg_occ_desc_init(dg_occ_desc *desc, uint32_t N, const double extent[3]);
/* Host: what Sec. 5.1 prescribes at a training iteration -- whether the grid is refreshed now (every 16th),
 * whether the warm-up rule for candidates applies (< 4096), the decay factor and the bit threshold. */
void dg_occ_schedule(uint64_t iteration, int *update_now, int *warmup, float *decay, float *threshold);
/* Candidate cells [i0, i0 + M) of one refresh and a random point in each (a refresh may be produced in several
 * calls): cell [M] uint32, u [M,3] fp32 (device).  A refresh has all n_cells cells as candidates during warm-up and
 * n_cells/2 afterwards, half of them uniform (Instant-NGP App. E.2).
 * warmup != 0: candidate i is cell i (i0 + M <= n_cells).  Otherwise candidates i < n_uniform are uniform draws over
 * all cells and the others are drawn among occupied cells by rejection: up to `tries` (1..64) uniform draws, the
 * first one whose bit is set, else the last.  Random numbers: splitmix64 output mix of
 * seed + 0x9E3779B97F4A7C15*(ctr+1), ctr = iteration<<36 | i<<8 | try<<2 | q (q = 0 cell, 1..3 position);
 * cell = (top 32 bits * n_cells) >> 32; u_d = (c_d + xi_d) / scale[d], xi = top 24 bits * 2^-24.
 * i0 + M <= 2^28, iteration < 2^28. */
int dg_occ_candidates(const dg_occ_desc *desc, const uint32_t *bits, uint32_t i0, uint32_t M, uint32_t n_uniform,
                      int warmup, uint64_t seed, uint32_t iteration, uint32_t tries, uint32_t *cell, float *u,
                      void *stream);
/* density[c] *= factor */
int dg_occ_decay(float *density, uint32_t n_cells, float factor, void *stream);
/* density[cell[i]] = max(density[cell[i]], sigma[i]); densities are >= 0, a sigma that is negative or NaN is ignored,
 * and so is a cell index >= n_cells */
int dg_occ_update(float *density, uint32_t n_cells, const uint32_t *cell, const float *sigma, uint32_t M,
                  void *stream);
/* bit of cell c = density[c] > threshold; *n_set (device, may be NULL) "+=" the number of set bits */
int dg_occ_bits(const float *density, uint32_t n_cells, float threshold, uint32_t *bits, uint32_t *n_set,
                void *stream);
/* Marching of the n_seg segments listed in seg_ray/seg_slot (as for dg_sample_segments) through box `box` (host,
 * 6 floats) with the occupancy bits of that box's sub-model.  A segment of length len = t_out - t_in is cut into
 * n = clamp(ceil(len / dt), 1, max_steps) equal strata (max_steps <= 65535), stratum s is sampled at
 * t = t_in + (s + xi) * (len / n) with the jitter generator of dg_sample_segments, and the sample is kept iff the
 * bit of its cell is set (fp32 throughout, one rounding per operation).
 * Outputs (device): first [n_seg + 1] -- the samples of segment j are [first[j], first[j+1]), first[n_seg] is the
 * total; u [capacity,3], delta [capacity] (stratum width), t [capacity], sample_ray [capacity] (ray of each sample,
 * the index for dg_dir_encode).  Samples at positions >= capacity are not written and bit 1 of *status is set: the
 * caller reads first[n_seg] back and must not use more than it has room for.
 * ws: dg_march_workspace_bytes(n_seg) bytes of device memory. */
size_t dg_march_workspace_bytes(uint32_t n_seg);
int dg_march_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                      const uint32_t *seg_slot, uint32_t n_seg, uint32_t k_max, const float *box,
                      const dg_occ_desc *occ, const uint32_t *bits, float dt, uint32_t max_steps, uint64_t seed,
                      uint32_t capacity, uint32_t *first, float *u, float *delta, float *t, uint32_t *sample_ray,
                      uint32_t *status, void *ws, size_t ws_bytes, void *stream);
/* Local volume rendering (Eq. 3) of segments of different lengths: as dg_composite_segment_fwd / _depth / _bwd, with
 * segment j owning samples [first[j], first[j+1]); a segment without samples gives C_k = 0, T_k = 1, D_k = 0. */
int dg_composite_ragged_fwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                            const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                            float *Ck, float *Tk, void *stream);
int dg_composite_ragged_depth(const float *sigma, const float *delta, const float *t, uint32_t n_seg,
                              const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                              float *Dk, void *stream);
int dg_composite_ragged_bwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                            const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                            const float *gCk, const float *gTk, float *dsigma, float *drgb, void *stream);

#ifdef __cplusplus
}
#endif
#endif
