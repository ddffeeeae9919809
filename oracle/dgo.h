/*
 * dgo.h -- CPU oracle for the DistGrid training hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded, double
 * precision restatement of what the hot path computes, written from the
 * paper (DistGrid, arXiv 2405.04416) and from the published Instant-NGP
 * equations the paper inherits.  It shares no code, header, table or
 * constant generator with the HIP library and must never be linked, imported
 * or called by it.  Only tests, the smoke check and the benchmark's
 * cpu-baseline leg may use it.
 *
 * All pointers are host pointers.  Arrays are row-major, innermost dimension
 * last.  Floating point inputs that the method fixes as fp32 (coordinates,
 * tables, ray data) are float; every result the oracle computes is double,
 * except the two places where the method demands bit-exact fp32/integer
 * bookkeeping (segment times and vertex indices).
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned to a
 * closed form, an invariant, a library routine or brute force; none is
 * "parity unpinned".  dgo_grid_param_count is pinned by brute force (every
 * vertex of every level of small grids visited, the reached entries counted)
 * and to the bound of Sec. 3.2; the two totals the paper prints (Sec. 5.3)
 * cannot be reproduced, the scenes' extents and base resolution are not given.
 */
#ifndef DGO_H
#define DGO_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DGO_MAX_LEVELS 16

/* Deformable multi-resolution hash grid geometry (Sec. 3.2, Sec. 4.1). */
typedef struct {
    uint32_t L;                         /* number of levels                       */
    uint32_t F;                         /* features per entry                     */
    uint32_t log2_T;                    /* hash table length T = 2^log2_T         */
    uint32_t N[DGO_MAX_LEVELS];         /* N_l: voxels along the longest axis     */
    uint32_t shape[DGO_MAX_LEVELS][3];  /* voxels per axis: ceil(a_d/s * N_l)     */
    uint32_t is_dense[DGO_MAX_LEVELS];  /* one-to-one map if #vertices <= T       */
    uint64_t first[DGO_MAX_LEVELS + 1]; /* first entry of each level in the table */
    float    gain[DGO_MAX_LEVELS][3];   /* grid position = u_d * gain[l][d]       */
} dgo_grid;

/* N_l = floor(N_min * b^l) (Instant-NGP Eq. 2), shape per Sec. 4.1. */
int dgo_grid_init(dgo_grid *g, uint32_t L, uint32_t F, uint32_t log2_T,
                  uint32_t N_min, double growth, const double extent[3]);
/* b = exp((ln N_max - ln N_min)/(L-1)) (Instant-NGP Eq. 3). */
double dgo_growth_factor(uint32_t N_min, uint32_t N_max, uint32_t L);
uint64_t dgo_grid_param_count(const dgo_grid *g);

/* Spatial hash of integer vertex coordinates (Instant-NGP Eq. 4), T = 2^log2_T. */
uint32_t dgo_hash(uint32_t x, uint32_t y, uint32_t z, uint32_t log2_T);
/* Entry index (relative to the level's first entry) of vertex (x,y,z). */
uint32_t dgo_vertex_entry(const dgo_grid *g, uint32_t level, uint32_t x, uint32_t y, uint32_t z);

/* Encode forward: feat[n, l*F+f] = sum over the 8 cell corners of w_c * table[entry_c, f].
 * idx (nullable) receives the absolute entry index of each corner: [N, L, 8]. */
void dgo_encode_fwd(const dgo_grid *g, const float *table, const float *u, uint64_t n,
                    double *feat, uint32_t *idx, int abs_terms);
/* Encode backward (transpose): dtable[entry_c, f] += w_c * dfeat[n, l*F+f]. */
void dgo_encode_bwd(const dgo_grid *g, const float *u, const double *dfeat, uint64_t n,
                    double *dtable);

/* Ray / AABB slab test against P boxes; ordered segment list per ray (Sec. 4.2.1, Fig. 2 step 2).
 * holes: NULL, or P boxes; partition p then covers its box minus holes[p] (the coarse level of the two-level
 * cascade of Sec. 4.2.2 covers the outer box around the inner one), which a ray meets in up to two segments. */
void dgo_ray_aabb_segments(const float *o, const float *d, uint32_t R, const float *aabb, const float *holes,
                           uint32_t P, float t_min, uint32_t k_max, uint32_t *seg_count, float *seg_t,
                           int32_t *seg_part, uint32_t *status);
/* Stable distribution of (ray, slot) pairs to partitions (Fig. 2 step 3). */
void dgo_bucket_segments(const uint32_t *seg_count, const int32_t *seg_part, uint32_t R, uint32_t k_max,
                         uint32_t P, uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot);
/* Counter-based jitter in [0,1) for (seed, ray, slot, sample). */
float dgo_jitter(uint64_t seed, uint32_t ray, uint32_t slot, uint32_t s);
/* Stratified samples of segments [seg_begin, seg_end) that all lie in box `aabb6`. */
void dgo_sample_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                         const uint32_t *seg_slot, uint32_t seg_begin, uint32_t seg_end, uint32_t k_max,
                         const float *aabb6, uint32_t S, uint64_t seed, const float *jitter,
                         float *u, float *delta, float *t /* nullable: sample distances */);

/* Real spherical harmonics, bands l = 0..degree-1, on normalised d: out [n, degree^2]. */
void dgo_sh(const float *d, uint64_t n, uint32_t degree, double *out);

/* fp16 round-to-nearest-even of a double, returned as double. */
double dgo_round_f16(double x);

/* Field MLP pair (density then colour, Sec. 3.2 / Sec. 5.1). */
typedef struct {
    uint32_t n_feat;      /* density input width (L*F)                        */
    uint32_t n_hidden_d;  /* density hidden width (one ReLU hidden layer)     */
    uint32_t n_geo;       /* density output width; out[0] is the raw density  */
    uint32_t n_dir;       /* direction-encoding width                         */
    uint32_t n_hidden_c;  /* colour hidden width                              */
    uint32_t n_layers_c;  /* colour hidden layers: 1 or 2                     */
    uint32_t act_c;       /* colour hidden activation: 0 ReLU, 1 sigmoid      */
    uint32_t round_f16;   /* 1: apply the fp16 rounding points; 0: pure double */
} dgo_mlp;
uint64_t dgo_mlp_weight_count(const dgo_mlp *m);
void dgo_mlp_fwd(const dgo_mlp *m, const double *w, const double *feat, const double *dir_enc,
                 uint32_t S, uint64_t n, double *sigma, double *rgb);
void dgo_mlp_bwd(const dgo_mlp *m, const double *w, const double *feat, const double *dir_enc,
                 uint32_t S, uint64_t n, const double *dsigma, const double *drgb, double loss_scale,
                 double *dfeat, double *dw);

/* Discrete volume rendering of one segment of S samples (Eq. 3 by quadrature). */
void dgo_composite_fwd(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                       uint32_t S, double *C, double *T);
void dgo_composite_bwd(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                       uint32_t S, const double *gC, const double *gT, double *dsigma, double *drgb);

/* Segmented volume rendering merge (Eq. 5, 6) and its backward (Eq. 7, 8). */
void dgo_merge_fwd(const double *Ck, const double *Tk, const uint32_t *seg_count, uint32_t R,
                   uint32_t k_max, double *C, double *T);
void dgo_merge_bwd(const double *Ck, const double *Tk, const uint32_t *seg_count, uint32_t R,
                   uint32_t k_max, const double *gC, const double *gT, double *gCk, double *gTk);

/* Loss (Eq. 9 as a mean, plus lambda1 * Eq. 10) and its gradient seeds. */
double dgo_loss(const double *C, const double *T, const double *Cgt, uint32_t R, double lambda1,
                double *gC, double *gT);

/* Depth for evaluation rendering (Sec. 4.4.2: colour, depth and transmittance are merged from the partial results): per segment
 * D_k = sum_i T_i alpha_i t_i, merged as D = sum_k (prod_{j<k} T_j) D_k, i.e. like colour under Eq. 5. */
void dgo_composite_depth(const double *sigma, const double *delta, const double *t, uint32_t n_seg, uint32_t S,
                         double *D);
void dgo_merge_depth(const double *Dk, const double *Tk, const uint32_t *seg_count, uint32_t R, uint32_t k_max,
                     double *D);

/* One Adam step (Kingma & Ba 2015, Algorithm 1; optimiser named in Sec. 5.1) on n parameters, in place:
 * g' = g + l2 * theta;  m = b1 m + (1-b1) g';  v = b2 v + (1-b2) g'^2;
 * theta -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = step >= 1.
 * skip_zero != 0: a parameter whose gradient is exactly 0 is left alone altogether (value and both moments), the
 * rule of the system whose unnamed hyper-parameters Sec. 5.1 inherits, for sparsely touched hash tables. */
void dgo_adam_step(double *theta, const double *grad, double *m, double *v, uint64_t n, double lr,
                   double beta1, double beta2, double eps, uint32_t step, double l2, int skip_zero);

/* Learning rate of Sec. 5.1: from lr0 down to lr1 along half a cosine over `total` iterations. */
double dgo_cosine_lr(double lr0, double lr1, uint64_t iteration, uint64_t total);

/* ------------------------------------------------------------------------------------------------
 * Occupancy grid and occupancy-guided sampling (Sec. 3.2: a grid of per-voxel densities lets ray
 * marching skip empty space; Sec. 4.1: it is deformable like the hash grid; Sec. 5.1: one scale, plain
 * x-fastest storage, resolution 512, decay 0.99 every 16 iterations, warm-up 4096 iterations, bit
 * threshold 0.6 before iteration 10 000 and 60 after; the update rule itself is Instant-NGP App. E.2).
 * Everything that decides an integer (a cell, a bit, a sample count) is computed in fp32 / integers.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    uint32_t shape[3];      /* cells per axis: ceil(a_d/s * N)                  */
    uint32_t n_cells;
    float    gain[3];       /* grid position of unit coordinate u_d: u_d * gain */
} dgo_occ;
int dgo_occ_init(dgo_occ *g, uint32_t N, const double extent[3]);
/* cell of a point with unit coordinates u (clamped to [0,1]): x + shape_x (y + shape_y z) */
uint32_t dgo_occ_cell(const dgo_occ *g, const float *u3);
/* when and how the grid is refreshed at a training iteration (Sec. 5.1) */
void dgo_occ_schedule(uint64_t iteration, int *update_now, int *warmup, float *decay, float *threshold);
/* 64 random bits for (seed, counter): splitmix64 output mix of seed + golden * (counter + 1) */
uint64_t dgo_rand64(uint64_t seed, uint64_t counter);
/* Candidate cells [i0, i0 + M) of one refresh (Instant-NGP App. E.2) and a random point inside each (a refresh may be
 * produced in several pieces).  warmup: candidate i is cell i (i0 + M <= n_cells).  Otherwise the first n_uniform candidates are
 * uniform draws over all cells and the others are drawn among the occupied cells by rejection: up to
 * `tries` uniform draws, the first whose bit is set wins, the last one is taken if none is.
 * Draw q (0 = cell, 1..3 = position) of try a of candidate i uses counter (iteration<<36)|(i<<8)|(a<<2)|q;
 * cell = (top 32 bits * n_cells) >> 32; position u_d = (c_d + xi_d) / gain_d, xi from the top 24 bits. */
void dgo_occ_candidates(const dgo_occ *g, const uint32_t *bits, uint32_t i0, uint32_t M, uint32_t n_uniform, int warmup,
                        uint64_t seed, uint32_t iteration, uint32_t tries, uint32_t *cell, float *u);
void dgo_occ_decay(float *density, uint32_t n_cells, float factor);
/* density[cell[i]] = max(density[cell[i]], sigma[i]) */
void dgo_occ_update(float *density, const uint32_t *cell, const float *sigma, uint32_t M);
/* bit (c % 32) of word c / 32 = density[c] > threshold; returns the number of set bits */
uint32_t dgo_occ_bits(const float *density, uint32_t n_cells, float threshold, uint32_t *bits);
/* Marching of the segments [seg_begin, seg_end) of one box: a segment of length len = t_out - t_in is cut
 * into n = clamp(ceil(len / dt), 1, max_steps) equal strata, stratum s is sampled at t_in + (s + xi) len/n
 * (xi as in dgo_sample_segments) and the sample is kept iff the bit of its cell is set.  first[j - seg_begin]
 * receives the number of samples kept before segment j (n_seg + 1 values).  The sample arrays may be NULL
 * (counting only).  Returns the total. */
uint32_t dgo_march_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                            const uint32_t *seg_slot, uint32_t seg_begin, uint32_t seg_end, uint32_t k_max,
                            const float *aabb6, const dgo_occ *g, const uint32_t *bits, float dt,
                            uint32_t max_steps, uint64_t seed, uint32_t *first, float *u, float *delta,
                            float *t, uint32_t *sample_ray);
/* Eq. 3 on segments of different lengths: segment j owns samples [first[j], first[j+1]) */
void dgo_composite_fwd_ragged(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                              const uint32_t *first, double *C, double *T);
void dgo_composite_bwd_ragged(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                              const uint32_t *first, const double *gC, const double *gT, double *dsigma,
                              double *drgb);
void dgo_composite_depth_ragged(const double *sigma, const double *delta, const double *t, uint32_t n_seg,
                                const uint32_t *first, double *D);

#ifdef __cplusplus
}
#endif
#endif
