/*
 * dgo.c -- CPU oracle for the DistGrid training hot path (see dgo.h).
 *
 * TEST INFRASTRUCTURE ONLY: never part of the product path.
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared dgo.c -lm
 * (-ffp-contract=off matters: the fp32 bookkeeping below must round after
 *  every operation so that it can be compared bit for bit.)
 */
#include "dgo.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Grid geometry (Sec. 3.2, Sec. 4.1; Instant-NGP Eq. 2-3)             */
/* ------------------------------------------------------------------ */

double dgo_growth_factor(uint32_t N_min, uint32_t N_max, uint32_t L)
{
    if (L < 2) return 1.0;
    return exp((log((double)N_max) - log((double)N_min)) / (double)(L - 1));
}

int dgo_grid_init(dgo_grid *g, uint32_t L, uint32_t F, uint32_t log2_T,
                  uint32_t N_min, double growth, const double extent[3])
{
    if (!g || L == 0 || L > DGO_MAX_LEVELS || F == 0 || log2_T > 28) return -1;
    memset(g, 0, sizeof *g);
    g->L = L; g->F = F; g->log2_T = log2_T;
    const uint64_t T = (uint64_t)1 << log2_T;
    double s = extent[0];
    if (extent[1] > s) s = extent[1];
    if (extent[2] > s) s = extent[2];
    if (!(s > 0.0)) return -1;
    uint64_t first = 0;
    for (uint32_t l = 0; l < L; ++l) {
        /* geometric growth; the small bias keeps an exactly-integer product
           (e.g. N_max at the top level) from falling one below through rounding */
        double Nl = floor((double)N_min * pow(growth, (double)l) + 1e-6);
        g->N[l] = (uint32_t)Nl;
        uint64_t verts = 1;
        for (int a = 0; a < 3; ++a) {
            double cells = extent[a] / s * Nl;          /* a/s * N_l, Sec. 4.1 */
            g->shape[l][a] = (uint32_t)ceil(cells);
            if (g->shape[l][a] == 0) g->shape[l][a] = 1;
            g->gain[l][a] = (float)cells;               /* cubic voxels of side s/N_l */
            verts *= (uint64_t)g->shape[l][a] + 1;
        }
        g->is_dense[l] = verts <= T;
        g->first[l] = first;
        uint64_t len = g->is_dense[l] ? ((verts + 7) / 8) * 8 : T;
        first += len;
    }
    g->first[L] = first;
    return 0;
}

uint64_t dgo_grid_param_count(const dgo_grid *g)
{
    return g->first[g->L] * g->F;
}

uint32_t dgo_hash(uint32_t x, uint32_t y, uint32_t z, uint32_t log2_T)
{
    /* xor of the coordinates times per-axis primes (first prime is 1), modulo T */
    const uint32_t p2 = 2654435761u, p3 = 805459861u;
    uint32_t h = x ^ (y * p2) ^ (z * p3);
    return (uint32_t)((uint64_t)h % ((uint64_t)1 << log2_T));
}

uint32_t dgo_vertex_entry(const dgo_grid *g, uint32_t level, uint32_t x, uint32_t y, uint32_t z)
{
    if (g->is_dense[level]) {
        uint32_t nx = g->shape[level][0] + 1, ny = g->shape[level][1] + 1;
        return x + nx * (y + ny * z);
    }
    return dgo_hash(x, y, z, g->log2_T);
}

/* cell of a sample at one level: lower corner and fractional offsets */
static void locate(const dgo_grid *g, uint32_t l, const float *u3, uint32_t cell[3], float frac[3])
{
    for (int a = 0; a < 3; ++a) {
        float u = u3[a];
        if (!(u >= 0.0f)) u = 0.0f;          /* also catches NaN */
        if (u > 1.0f) u = 1.0f;
        float pos = u * g->gain[l][a];       /* one fp32 multiply */
        float fl = floorf(pos);
        uint32_t i = (uint32_t)fl;
        uint32_t last = g->shape[l][a] - 1;
        if (i > last) i = last;              /* u == 1 lands in the last cell */
        cell[a] = i;
        frac[a] = pos - (float)i;            /* exact in fp32 */
    }
}

void dgo_encode_fwd(const dgo_grid *g, const float *table, const float *u, uint64_t n,
                    double *feat, uint32_t *idx, int abs_terms)
{
    const uint32_t L = g->L, F = g->F;
    for (uint64_t i = 0; i < n; ++i) {
        for (uint32_t l = 0; l < L; ++l) {
            uint32_t cell[3]; float frac[3];
            locate(g, l, u + 3 * i, cell, frac);
            double acc[8] = {0};
            for (uint32_t c = 0; c < 8; ++c) {
                uint32_t cx = c & 1, cy = (c >> 1) & 1, cz = (c >> 2) & 1;
                double w = (cx ? (double)frac[0] : 1.0 - (double)frac[0]) *
                           (cy ? (double)frac[1] : 1.0 - (double)frac[1]) *
                           (cz ? (double)frac[2] : 1.0 - (double)frac[2]);
                uint64_t e = g->first[l] + dgo_vertex_entry(g, l, cell[0] + cx, cell[1] + cy, cell[2] + cz);
                if (idx) idx[(i * L + l) * 8 + c] = (uint32_t)e;
                for (uint32_t f = 0; f < F; ++f) {
                    double v = (double)table[e * F + f];
                    acc[f] += w * (abs_terms ? fabs(v) : v);
                }
            }
            for (uint32_t f = 0; f < F; ++f) feat[i * L * F + l * F + f] = acc[f];
        }
    }
}

void dgo_encode_bwd(const dgo_grid *g, const float *u, const double *dfeat, uint64_t n,
                    double *dtable)
{
    const uint32_t L = g->L, F = g->F;
    for (uint64_t i = 0; i < n; ++i) {
        for (uint32_t l = 0; l < L; ++l) {
            uint32_t cell[3]; float frac[3];
            locate(g, l, u + 3 * i, cell, frac);
            for (uint32_t c = 0; c < 8; ++c) {
                uint32_t cx = c & 1, cy = (c >> 1) & 1, cz = (c >> 2) & 1;
                double w = (cx ? (double)frac[0] : 1.0 - (double)frac[0]) *
                           (cy ? (double)frac[1] : 1.0 - (double)frac[1]) *
                           (cz ? (double)frac[2] : 1.0 - (double)frac[2]);
                uint64_t e = g->first[l] + dgo_vertex_entry(g, l, cell[0] + cx, cell[1] + cy, cell[2] + cz);
                for (uint32_t f = 0; f < F; ++f)
                    dtable[e * F + f] += w * dfeat[i * L * F + l * F + f];
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Rays, boxes, segments (Sec. 4.2.1, Sec. 4.4.2, Fig. 2 steps 2-3)    */
/* ------------------------------------------------------------------ */

/* slab test of one ray against one box; 0 = miss.  One rounding per operation; a ray parallel to a slab is inside
 * iff lo <= o < hi (half-open, so a ray lying in a shared face belongs to the higher box). */
static int slab_interval(const float *o, const float *d, const float *lo, const float *hi, float t_min,
                         float *t_in, float *t_out)
{
    float tn = -INFINITY, tf = INFINITY;
    for (int a = 0; a < 3; ++a) {
        float oa = o[a], da = d[a];
        if (da == 0.0f) {
            if (!(lo[a] <= oa && oa < hi[a])) return 0;
            continue;
        }
        float inv = 1.0f / da;
        float t1 = (lo[a] - oa) * inv;
        float t2 = (hi[a] - oa) * inv;
        tn = fmaxf(tn, fminf(t1, t2));
        tf = fminf(tf, fmaxf(t1, t2));
    }
    *t_in = fmaxf(tn, t_min);
    *t_out = tf;
    return *t_out > *t_in;
}

/* insert a segment in front-to-back order: ascending entry time, ties keep the order of insertion */
static void insert_segment(float *st, int32_t *sp, uint32_t *cnt, uint32_t k_max, uint32_t *status,
                           float t_in, float t_out, int32_t p)
{
    uint32_t pos = *cnt < k_max ? *cnt : k_max;
    while (pos > 0 && st[2 * (pos - 1)] > t_in) --pos;
    if (pos >= k_max) { if (status) *status |= 1u; return; }
    if (*cnt >= k_max && status) *status |= 1u;
    uint32_t last = *cnt < k_max ? *cnt : k_max - 1;
    for (uint32_t k = last; k > pos; --k) {
        st[2 * k] = st[2 * (k - 1)]; st[2 * k + 1] = st[2 * (k - 1) + 1]; sp[k] = sp[k - 1];
    }
    st[2 * pos] = t_in; st[2 * pos + 1] = t_out; sp[pos] = p;
    if (*cnt < k_max) ++*cnt;
}

void dgo_ray_aabb_segments(const float *o, const float *d, uint32_t R, const float *aabb, const float *holes,
                           uint32_t P, float t_min, uint32_t k_max, uint32_t *seg_count, float *seg_t,
                           int32_t *seg_part, uint32_t *status)
{
    for (uint32_t r = 0; r < R; ++r) {
        uint32_t cnt = 0;
        float *st = seg_t + (uint64_t)r * k_max * 2;
        int32_t *sp = seg_part + (uint64_t)r * k_max;
        for (uint32_t k = 0; k < k_max; ++k) { st[2 * k] = 0.0f; st[2 * k + 1] = 0.0f; sp[k] = -1; }
        for (uint32_t p = 0; p < P; ++p) {
            const float *lo = aabb + 6 * p, *hi = lo + 3;
            float t_in, t_out;
            if (!slab_interval(o + 3 * r, d + 3 * r, lo, hi, t_min, &t_in, &t_out)) continue;
            /* the region of partition p is its box minus its hole (Sec. 4.2.2: the coarse level covers the outer box
             * around the inner one); a hole with no volume is no hole */
            const float *hlo = holes ? holes + 6 * p : NULL, *hhi = hlo ? hlo + 3 : NULL;
            float h_in, h_out;
            if (hlo && hhi[0] > hlo[0] && hhi[1] > hlo[1] && hhi[2] > hlo[2] &&
                slab_interval(o + 3 * r, d + 3 * r, hlo, hhi, t_min, &h_in, &h_out)) {
                /* the hole may reach beyond the box: both pieces stay inside the box's own interval */
                float first_end = fminf(h_in, t_out), second_begin = fmaxf(h_out, t_in);
                if (first_end > t_in) insert_segment(st, sp, &cnt, k_max, status, t_in, first_end, (int32_t)p);
                if (t_out > second_begin) insert_segment(st, sp, &cnt, k_max, status, second_begin, t_out, (int32_t)p);
            } else {
                insert_segment(st, sp, &cnt, k_max, status, t_in, t_out, (int32_t)p);
            }
        }
        seg_count[r] = cnt;
    }
}

void dgo_bucket_segments(const uint32_t *seg_count, const int32_t *seg_part, uint32_t R, uint32_t k_max,
                         uint32_t P, uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot)
{
    for (uint32_t p = 0; p <= P; ++p) part_offset[p] = 0;
    for (uint32_t r = 0; r < R; ++r)
        for (uint32_t k = 0; k < seg_count[r]; ++k)
            part_offset[seg_part[(uint64_t)r * k_max + k] + 1]++;
    for (uint32_t p = 0; p < P; ++p) part_offset[p + 1] += part_offset[p];
    uint32_t *cursor = (uint32_t *)malloc(sizeof(uint32_t) * (P ? P : 1));
    for (uint32_t p = 0; p < P; ++p) cursor[p] = part_offset[p];
    for (uint32_t r = 0; r < R; ++r)
        for (uint32_t k = 0; k < seg_count[r]; ++k) {
            uint32_t p = (uint32_t)seg_part[(uint64_t)r * k_max + k];
            seg_ray[cursor[p]] = r; seg_slot[cursor[p]] = k; cursor[p]++;
        }
    free(cursor);
}

float dgo_jitter(uint64_t seed, uint32_t ray, uint32_t slot, uint32_t s)
{
    /* counter-based: a 64-bit counter pushed through the splitmix64 output mix */
    uint64_t ctr = ((uint64_t)ray << 32) | ((uint64_t)(slot & 0xffffu) << 16) | (uint64_t)(s & 0xffffu);
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (ctr + 1);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    return (float)(z >> 40) * (1.0f / 16777216.0f);
}

void dgo_sample_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                         const uint32_t *seg_slot, uint32_t seg_begin, uint32_t seg_end, uint32_t k_max,
                         const float *aabb6, uint32_t S, uint64_t seed, const float *jitter,
                         float *u, float *delta, float *t_out_samples)
{
    float inv_ext[3];
    for (int a = 0; a < 3; ++a) inv_ext[a] = 1.0f / (aabb6[3 + a] - aabb6[a]);
    for (uint32_t j = seg_begin; j < seg_end; ++j) {
        uint32_t r = seg_ray[j], k = seg_slot[j];
        float t_in = seg_t[((uint64_t)r * k_max + k) * 2], t_out = seg_t[((uint64_t)r * k_max + k) * 2 + 1];
        float dt = (t_out - t_in) / (float)S;      /* stratum width */
        for (uint32_t s = 0; s < S; ++s) {
            uint64_t n = (uint64_t)(j - seg_begin) * S + s;
            float xi = jitter ? jitter[n] : dgo_jitter(seed, r, k, s);
            float t = t_in + ((float)s + xi) * dt;
            for (int a = 0; a < 3; ++a) {
                float x = fmaf(t, d[3 * r + a], o[3 * r + a]);
                u[3 * n + a] = (x - aabb6[a]) * inv_ext[a];
            }
            delta[n] = dt;
            if (t_out_samples) t_out_samples[n] = t;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Direction encoding: real spherical harmonics from their definition  */
/* ------------------------------------------------------------------ */

static double factorial(int n) { double f = 1.0; for (int i = 2; i <= n; ++i) f *= i; return f; }

/* associated Legendre P_l^m(x), m >= 0, with the Condon-Shortley phase */
static double legendre(int l, int m, double x)
{
    double pmm = 1.0;
    if (m > 0) {
        double somx2 = sqrt((1.0 - x) * (1.0 + x));
        double fact = 1.0;
        for (int i = 1; i <= m; ++i) { pmm *= -fact * somx2; fact += 2.0; }
    }
    if (l == m) return pmm;
    double pmmp1 = x * (2.0 * m + 1.0) * pmm;
    if (l == m + 1) return pmmp1;
    double pll = 0.0;
    for (int ll = m + 2; ll <= l; ++ll) {
        pll = ((2.0 * ll - 1.0) * x * pmmp1 - (ll + m - 1.0) * pmm) / (ll - m);
        pmm = pmmp1; pmmp1 = pll;
    }
    return pll;
}

void dgo_sh(const float *d, uint64_t n, uint32_t degree, double *out)
{
    const double PI = 3.14159265358979323846;
    for (uint64_t i = 0; i < n; ++i) {
        double x = d[3 * i], y = d[3 * i + 1], z = d[3 * i + 2];
        double r = sqrt(x * x + y * y + z * z);
        double ct = r > 0 ? z / r : 1.0;
        if (ct > 1.0) ct = 1.0;
        if (ct < -1.0) ct = -1.0;
        double phi = atan2(y, x);
        for (int l = 0; l < (int)degree; ++l) {
            for (int m = -l; m <= l; ++m) {
                int am = m < 0 ? -m : m;
                double K = sqrt((2.0 * l + 1.0) / (4.0 * PI) * factorial(l - am) / factorial(l + am));
                double v;
                if (m == 0) v = K * legendre(l, 0, ct);
                else if (m > 0) v = sqrt(2.0) * K * cos(m * phi) * legendre(l, m, ct);
                else v = sqrt(2.0) * K * sin(am * phi) * legendre(l, am, ct);
                out[i * degree * degree + (uint64_t)(l * l + l + m)] = v;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Field MLPs (Sec. 3.2: a small fusing MLP; Sec. 5.1 activations, clip) */
/* ------------------------------------------------------------------ */

double dgo_round_f16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    double a = fabs(x);
    int e;
    frexp(a, &e);              /* a = m * 2^e, m in [0.5,1)  => floor(log2 a) = e-1 */
    int p = e - 1;
    double q = p < -14 ? ldexp(1.0, -24) : ldexp(1.0, p - 10);  /* spacing of fp16 at a */
    double r = nearbyint(a / q) * q;                            /* ties to even */
    if (r >= 65520.0) r = INFINITY;
    return copysign(r, x);
}

uint64_t dgo_mlp_weight_count(const dgo_mlp *m)
{
    uint64_t c = (uint64_t)m->n_hidden_d * m->n_feat + (uint64_t)m->n_geo * m->n_hidden_d;
    c += (uint64_t)m->n_hidden_c * (m->n_geo + m->n_dir);
    if (m->n_layers_c == 2) c += (uint64_t)m->n_hidden_c * m->n_hidden_c;
    c += 3ull * m->n_hidden_c;
    return c;
}

typedef struct { const double *Wd1, *Wd2, *Wc1, *Wc2, *Wc3; } weights_view;
static weights_view view(const dgo_mlp *m, const double *w)
{
    weights_view v;
    v.Wd1 = w;
    v.Wd2 = v.Wd1 + (uint64_t)m->n_hidden_d * m->n_feat;
    v.Wc1 = v.Wd2 + (uint64_t)m->n_geo * m->n_hidden_d;
    const double *next = v.Wc1 + (uint64_t)m->n_hidden_c * (m->n_geo + m->n_dir);
    if (m->n_layers_c == 2) { v.Wc2 = next; next += (uint64_t)m->n_hidden_c * m->n_hidden_c; }
    else v.Wc2 = 0;
    v.Wc3 = next;
    return v;
}

#define MAXW 256
static double rnd(const dgo_mlp *m, double x) { return m->round_f16 ? dgo_round_f16(x) : x; }
static double clip15(double x) { return x < -15.0 ? -15.0 : (x > 15.0 ? 15.0 : x); }
static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }
static double act(uint32_t kind, double x) { return kind ? sigmoid(x) : (x > 0.0 ? x : 0.0); }
/* derivative expressed through the (rounded) activation value a */
static double dact(uint32_t kind, double a) { return kind ? a * (1.0 - a) : (a > 0.0 ? 1.0 : 0.0); }

/* y[o] = sum_i W[o,i] x[i] */
static void matvec(const double *W, uint32_t n_out, uint32_t n_in, const double *x, double *y)
{
    for (uint32_t o = 0; o < n_out; ++o) {
        double s = 0.0;
        for (uint32_t i = 0; i < n_in; ++i) s += W[(uint64_t)o * n_in + i] * x[i];
        y[o] = s;
    }
}
/* x[i] = sum_o W[o,i] y[o] */
static void matvec_t(const double *W, uint32_t n_out, uint32_t n_in, const double *y, double *x)
{
    for (uint32_t i = 0; i < n_in; ++i) {
        double s = 0.0;
        for (uint32_t o = 0; o < n_out; ++o) s += W[(uint64_t)o * n_in + i] * y[o];
        x[i] = s;
    }
}
/* dW[o,i] += y[o] * x[i] * scale */
static void outer_acc(double *dW, uint32_t n_out, uint32_t n_in, const double *y, const double *x, double scale)
{
    for (uint32_t o = 0; o < n_out; ++o)
        for (uint32_t i = 0; i < n_in; ++i) dW[(uint64_t)o * n_in + i] += y[o] * x[i] * scale;
}

typedef struct {
    double x0[MAXW], h1[MAXW], geo[MAXW], xc[MAXW], c1[MAXW], c2[MAXW], raw[3], sigma, rgb[3];
} activations;

static void forward_one(const dgo_mlp *m, const weights_view *v, const double *feat, const double *dir,
                        activations *a)
{
    const uint32_t nc_in = m->n_geo + m->n_dir;
    double z[MAXW];
    for (uint32_t i = 0; i < m->n_feat; ++i) a->x0[i] = rnd(m, feat[i]);
    matvec(v->Wd1, m->n_hidden_d, m->n_feat, a->x0, z);
    for (uint32_t i = 0; i < m->n_hidden_d; ++i) a->h1[i] = rnd(m, act(0, z[i]));
    matvec(v->Wd2, m->n_geo, m->n_hidden_d, a->h1, a->geo);
    a->sigma = exp(clip15(a->geo[0]));
    for (uint32_t i = 0; i < m->n_geo; ++i) a->xc[i] = rnd(m, a->geo[i]);
    for (uint32_t i = 0; i < m->n_dir; ++i) a->xc[m->n_geo + i] = rnd(m, dir[i]);
    matvec(v->Wc1, m->n_hidden_c, nc_in, a->xc, z);
    for (uint32_t i = 0; i < m->n_hidden_c; ++i) a->c1[i] = rnd(m, act(m->act_c, z[i]));
    const double *last = a->c1;
    if (m->n_layers_c == 2) {
        matvec(v->Wc2, m->n_hidden_c, m->n_hidden_c, a->c1, z);
        for (uint32_t i = 0; i < m->n_hidden_c; ++i) a->c2[i] = rnd(m, act(m->act_c, z[i]));
        last = a->c2;
    }
    matvec(v->Wc3, 3, m->n_hidden_c, last, a->raw);
    for (int c = 0; c < 3; ++c) a->rgb[c] = sigmoid(clip15(a->raw[c]));
}

void dgo_mlp_fwd(const dgo_mlp *m, const double *w, const double *feat, const double *dir_enc,
                 uint32_t S, uint64_t n, double *sigma, double *rgb)
{
    weights_view v = view(m, w);
    activations a;
    for (uint64_t i = 0; i < n; ++i) {
        forward_one(m, &v, feat + i * m->n_feat, dir_enc + (i / S) * m->n_dir, &a);
        sigma[i] = a.sigma;
        for (int c = 0; c < 3; ++c) rgb[3 * i + c] = a.rgb[c];
    }
}

void dgo_mlp_bwd(const dgo_mlp *m, const double *w, const double *feat, const double *dir_enc,
                 uint32_t S, uint64_t n, const double *dsigma, const double *drgb, double loss_scale,
                 double *dfeat, double *dw)
{
    weights_view v = view(m, w);
    /* gradient blocks in the same packing as the weights */
    double *dWd1 = dw + (v.Wd1 - w), *dWd2 = dw + (v.Wd2 - w), *dWc1 = dw + (v.Wc1 - w);
    double *dWc2 = v.Wc2 ? dw + (v.Wc2 - w) : 0, *dWc3 = dw + (v.Wc3 - w);
    const uint32_t nc_in = m->n_geo + m->n_dir;
    const double inv_scale = 1.0 / loss_scale;
    activations a;
    for (uint64_t i = 0; i < n; ++i) {
        forward_one(m, &v, feat + i * m->n_feat, dir_enc + (i / S) * m->n_dir, &a);
        double d3[3], g[MAXW], dl2[MAXW], dl1[MAXW], dgeo[MAXW], dh[MAXW];
        /* output sigmoid behind the [-15,15] clip */
        for (int c = 0; c < 3; ++c) {
            double pass = (a.raw[c] >= -15.0 && a.raw[c] <= 15.0) ? 1.0 : 0.0;
            d3[c] = rnd(m, loss_scale * drgb[3 * i + c] * a.rgb[c] * (1.0 - a.rgb[c]) * pass);
        }
        const double *last = m->n_layers_c == 2 ? a.c2 : a.c1;
        outer_acc(dWc3, 3, m->n_hidden_c, d3, last, inv_scale);
        matvec_t(v.Wc3, 3, m->n_hidden_c, d3, g);
        if (m->n_layers_c == 2) {
            for (uint32_t k = 0; k < m->n_hidden_c; ++k) dl2[k] = rnd(m, g[k] * dact(m->act_c, a.c2[k]));
            outer_acc(dWc2, m->n_hidden_c, m->n_hidden_c, dl2, a.c1, inv_scale);
            matvec_t(v.Wc2, m->n_hidden_c, m->n_hidden_c, dl2, g);
        }
        for (uint32_t k = 0; k < m->n_hidden_c; ++k) dl1[k] = rnd(m, g[k] * dact(m->act_c, a.c1[k]));
        outer_acc(dWc1, m->n_hidden_c, nc_in, dl1, a.xc, inv_scale);
        matvec_t(v.Wc1, m->n_hidden_c, nc_in, dl1, g);   /* only the first n_geo entries are used */
        /* density output: geometry features feed the colour net, out[0] also feeds exp() */
        double pass0 = (a.geo[0] >= -15.0 && a.geo[0] <= 15.0) ? 1.0 : 0.0;
        g[0] += loss_scale * dsigma[i] * a.sigma * pass0;
        for (uint32_t k = 0; k < m->n_geo; ++k) dgeo[k] = rnd(m, g[k]);
        outer_acc(dWd2, m->n_geo, m->n_hidden_d, dgeo, a.h1, inv_scale);
        matvec_t(v.Wd2, m->n_geo, m->n_hidden_d, dgeo, g);
        for (uint32_t k = 0; k < m->n_hidden_d; ++k) dh[k] = rnd(m, g[k] * dact(0, a.h1[k]));
        outer_acc(dWd1, m->n_hidden_d, m->n_feat, dh, a.x0, inv_scale);
        matvec_t(v.Wd1, m->n_hidden_d, m->n_feat, dh, g);
        for (uint32_t k = 0; k < m->n_feat; ++k) dfeat[i * m->n_feat + k] = g[k] * inv_scale;
    }
}

/* ------------------------------------------------------------------ */
/* Volume rendering of one segment (Eq. 3 by the standard quadrature)  */
/* ------------------------------------------------------------------ */

void dgo_composite_fwd(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                       uint32_t S, double *C, double *T)
{
    for (uint32_t j = 0; j < n_seg; ++j) {
        double trans = 1.0, col[3] = {0, 0, 0};
        for (uint32_t s = 0; s < S; ++s) {
            uint64_t n = (uint64_t)j * S + s;
            /* alpha = 1 - exp(-sigma delta); its complement is taken as exp(-sigma delta) itself,
               not as 1 - alpha, which cancels to nothing in double once sigma*delta > 36 */
            double keep = exp(-sigma[n] * delta[n]);
            double alpha = -expm1(-sigma[n] * delta[n]);
            double wgt = trans * alpha;
            for (int c = 0; c < 3; ++c) col[c] += wgt * rgb[3 * n + c];
            trans *= keep;
        }
        for (int c = 0; c < 3; ++c) C[3 * j + c] = col[c];
        T[j] = trans;
    }
}

void dgo_composite_bwd(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                       uint32_t S, const double *gC, const double *gT, double *dsigma, double *drgb)
{
    double *trans_before = (double *)malloc(sizeof(double) * (S + 1));
    for (uint32_t j = 0; j < n_seg; ++j) {
        trans_before[0] = 1.0;
        for (uint32_t s = 0; s < S; ++s) {
            uint64_t n = (uint64_t)j * S + s;
            trans_before[s + 1] = trans_before[s] * exp(-sigma[n] * delta[n]);
        }
        const double Tk = trans_before[S];
        /* behind[c] = sum over samples after s of w_j c_j : everything sample s shadows */
        double behind[3] = {0, 0, 0};
        for (uint32_t s = S; s-- > 0;) {
            uint64_t n = (uint64_t)j * S + s;
            double keep = exp(-sigma[n] * delta[n]);     /* 1 - alpha_s */
            double wgt = trans_before[s] * -expm1(-sigma[n] * delta[n]);
            double ds = 0.0;
            for (int c = 0; c < 3; ++c) {
                drgb[3 * n + c] = wgt * gC[3 * j + c];
                /* d alpha_s/d sigma_s = delta*keep raises w_s; every later weight scales by -delta */
                ds += gC[3 * j + c] * (trans_before[s] * keep * rgb[3 * n + c] - behind[c]);
            }
            ds -= gT[j] * Tk;
            dsigma[n] = delta[n] * ds;
            for (int c = 0; c < 3; ++c) behind[c] += wgt * rgb[3 * n + c];
        }
    }
    free(trans_before);
}

/* ------------------------------------------------------------------ */
/* Segmented volume rendering (Eq. 5-8)                                */
/* ------------------------------------------------------------------ */

void dgo_merge_fwd(const double *Ck, const double *Tk, const uint32_t *seg_count, uint32_t R,
                   uint32_t k_max, double *C, double *T)
{
    for (uint32_t r = 0; r < R; ++r) {
        uint32_t K = seg_count[r];
        const double *c = Ck + (uint64_t)r * k_max * 3, *t = Tk + (uint64_t)r * k_max;
        for (int ch = 0; ch < 3; ++ch) {
            double sum = 0.0;
            for (uint32_t i = 0; i < K; ++i) {
                double front = 1.0;                       /* T(t_-1,t_0) = 1 */
                for (uint32_t jx = 0; jx < i; ++jx) front *= t[jx];
                sum += front * c[3 * i + ch];
            }
            C[3 * r + ch] = sum;
        }
        double all = 1.0;
        for (uint32_t i = 0; i < K; ++i) all *= t[i];
        T[r] = all;
    }
}

void dgo_merge_bwd(const double *Ck, const double *Tk, const uint32_t *seg_count, uint32_t R,
                   uint32_t k_max, const double *gC, const double *gT, double *gCk, double *gTk)
{
    for (uint32_t r = 0; r < R; ++r) {
        uint32_t K = seg_count[r];
        const double *c = Ck + (uint64_t)r * k_max * 3, *t = Tk + (uint64_t)r * k_max;
        for (uint32_t i = 0; i < k_max; ++i) {
            for (int ch = 0; ch < 3; ++ch) gCk[((uint64_t)r * k_max + i) * 3 + ch] = 0.0;
            gTk[(uint64_t)r * k_max + i] = 0.0;
        }
        for (uint32_t i = 0; i < K; ++i) {
            /* Eq. 7 */
            double front = 1.0;
            for (uint32_t jx = 0; jx < i; ++jx) front *= t[jx];
            for (int ch = 0; ch < 3; ++ch) gCk[((uint64_t)r * k_max + i) * 3 + ch] = gC[3 * r + ch] * front;
            /* Eq. 8, products skip the factor j == i */
            double others = 1.0;
            for (uint32_t jx = 0; jx < K; ++jx) if (jx != i) others *= t[jx];
            double g = gT[r] * others;
            for (uint32_t k = i + 1; k < K; ++k) {
                double pr = 1.0;
                for (uint32_t jx = 0; jx < k; ++jx) if (jx != i) pr *= t[jx];
                for (int ch = 0; ch < 3; ++ch) g += gC[3 * r + ch] * pr * c[3 * k + ch];
            }
            gTk[(uint64_t)r * k_max + i] = g;
        }
    }
}

double dgo_loss(const double *C, const double *T, const double *Cgt, uint32_t R, double lambda1,
                double *gC, double *gT)
{
    double loss = 0.0;
    for (uint32_t r = 0; r < R; ++r) {
        for (int ch = 0; ch < 3; ++ch) {
            double e = C[3 * r + ch] - Cgt[3 * r + ch];
            loss += e * e / R;
            if (gC) gC[3 * r + ch] = 2.0 * e / R;
        }
        double opaque = 1.0 - T[r];
        if (opaque < 1e-6) opaque = 1e-6;
        loss += lambda1 * -log(opaque) / R;
        if (gT) gT[r] = (1.0 - T[r] >= 1e-6) ? lambda1 / (R * opaque) : 0.0;
    }
    return loss;
}

void dgo_adam_step(double *theta, const double *grad, double *m, double *v, uint64_t n, double lr,
                   double beta1, double beta2, double eps, uint32_t step, double l2, int skip_zero)
{
    const double c1 = 1.0 - pow(beta1, (double)step), c2 = 1.0 - pow(beta2, (double)step);
    for (uint64_t i = 0; i < n; ++i) {
        if (skip_zero && grad[i] == 0.0) continue;
        const double g = grad[i] + l2 * theta[i];
        m[i] = beta1 * m[i] + (1.0 - beta1) * g;
        v[i] = beta2 * v[i] + (1.0 - beta2) * g * g;
        const double m_hat = m[i] / c1, v_hat = v[i] / c2;
        theta[i] -= lr * m_hat / (sqrt(v_hat) + eps);
    }
}

double dgo_cosine_lr(double lr0, double lr1, uint64_t iteration, uint64_t total)
{
    const double pi = 3.14159265358979323846;
    const double x = iteration >= total ? 1.0 : (double)iteration / (double)total;
    return lr1 + 0.5 * (lr0 - lr1) * (1.0 + cos(pi * x));
}

/* Depth of evaluation rendering (Sec. 4.4.2: colour, depth and transmittance are merged): per segment the expected
 * distance sum_i T_i alpha_i t_i with the weights of Eq. 3's quadrature; merged like colour under Eq. 5. */
void dgo_composite_depth(const double *sigma, const double *delta, const double *t, uint32_t n_seg, uint32_t S,
                         double *D)
{
    for (uint32_t j = 0; j < n_seg; ++j) {
        double trans = 1.0, depth = 0.0;
        for (uint32_t s = 0; s < S; ++s) {
            uint64_t n = (uint64_t)j * S + s;
            depth += trans * -expm1(-sigma[n] * delta[n]) * t[n];
            trans *= exp(-sigma[n] * delta[n]);
        }
        D[j] = depth;
    }
}

void dgo_merge_depth(const double *Dk, const double *Tk, const uint32_t *seg_count, uint32_t R, uint32_t k_max,
                     double *D)
{
    for (uint32_t r = 0; r < R; ++r) {
        double sum = 0.0;
        for (uint32_t i = 0; i < seg_count[r]; ++i) {
            double front = 1.0;
            for (uint32_t jx = 0; jx < i; ++jx) front *= Tk[(uint64_t)r * k_max + jx];
            sum += front * Dk[(uint64_t)r * k_max + i];
        }
        D[r] = sum;
    }
}

/* ------------------------------------------------------------------ */
/* Occupancy grid and occupancy-guided sampling                        */
/* (Sec. 3.2, Sec. 4.1, Sec. 5.1; update rule: Instant-NGP App. E.2)   */
/* ------------------------------------------------------------------ */

int dgo_occ_init(dgo_occ *g, uint32_t N, const double extent[3])
{
    if (!g || N == 0) return -1;
    double s = extent[0];
    if (extent[1] > s) s = extent[1];
    if (extent[2] > s) s = extent[2];
    if (!(s > 0.0)) return -1;
    uint64_t cells = 1;
    for (int a = 0; a < 3; ++a) {
        if (!(extent[a] > 0.0)) return -1;
        double along = extent[a] / s * (double)N;       /* the hash grid's rule (Sec. 4.1) at one resolution */
        g->shape[a] = (uint32_t)ceil(along);
        if (g->shape[a] == 0) g->shape[a] = 1;
        g->gain[a] = (float)along;
        cells *= g->shape[a];
    }
    if (cells > 0xffffffffull) return -1;
    g->n_cells = (uint32_t)cells;
    return 0;
}

uint32_t dgo_occ_cell(const dgo_occ *g, const float *u3)
{
    uint32_t c[3];
    for (int a = 0; a < 3; ++a) {
        float v = u3[a];
        v = v >= 0.0f ? v : 0.0f;
        v = v > 1.0f ? 1.0f : v;
        float pos = v * g->gain[a];
        uint32_t i = (uint32_t)floorf(pos);
        if (i > g->shape[a] - 1) i = g->shape[a] - 1;
        c[a] = i;
    }
    return c[0] + g->shape[0] * (c[1] + g->shape[1] * c[2]);
}

void dgo_occ_schedule(uint64_t iteration, int *update_now, int *warmup, float *decay, float *threshold)
{
    *update_now = iteration % 16 == 0;          /* refreshed every 16 training iterations */
    *warmup = iteration < 4096;                 /* all cells are candidates during warm-up */
    *decay = 0.99f;
    *threshold = iteration < 10000 ? 0.6f : 60.0f;
}

uint64_t dgo_rand64(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (counter + 1);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static uint64_t candidate_counter(uint32_t iteration, uint32_t i, uint32_t attempt, uint32_t q)
{
    return ((uint64_t)iteration << 36) | ((uint64_t)i << 8) | ((uint64_t)attempt << 2) | q;
}

void dgo_occ_candidates(const dgo_occ *g, const uint32_t *bits, uint32_t i0, uint32_t M, uint32_t n_uniform, int warmup,
                        uint64_t seed, uint32_t iteration, uint32_t tries, uint32_t *cell, float *u)
{
    for (uint32_t i = i0; i < i0 + M; ++i) {
        uint32_t c = i, attempt = 0;
        if (!warmup) {
            uint32_t allowed = i < n_uniform ? 1 : tries;
            for (attempt = 0; attempt < allowed; ++attempt) {
                uint64_t z = dgo_rand64(seed, candidate_counter(iteration, i, attempt, 0));
                c = (uint32_t)(((z >> 32) * (uint64_t)g->n_cells) >> 32);
                if (i < n_uniform || ((bits[c >> 5] >> (c & 31)) & 1u)) break;
            }
            if (attempt == allowed) attempt = allowed - 1;      /* no occupied cell met: keep the last draw */
        }
        cell[i - i0] = c;
        uint32_t idx[3] = {c % g->shape[0], (c / g->shape[0]) % g->shape[1], c / (g->shape[0] * g->shape[1])};
        for (uint32_t a = 0; a < 3; ++a) {
            uint64_t z = dgo_rand64(seed, candidate_counter(iteration, i, attempt, a + 1));
            float xi = (float)(z >> 40) * (1.0f / 16777216.0f);
            u[3 * (uint64_t)(i - i0) + a] = ((float)idx[a] + xi) / g->gain[a];
        }
    }
}

void dgo_occ_decay(float *density, uint32_t n_cells, float factor)
{
    for (uint32_t c = 0; c < n_cells; ++c) density[c] = density[c] * factor;
}

void dgo_occ_update(float *density, const uint32_t *cell, const float *sigma, uint32_t M)
{
    for (uint32_t i = 0; i < M; ++i)
        if (sigma[i] > density[cell[i]]) density[cell[i]] = sigma[i];
}

uint32_t dgo_occ_bits(const float *density, uint32_t n_cells, float threshold, uint32_t *bits)
{
    uint32_t set = 0;
    for (uint32_t w = 0; w < (n_cells + 31) / 32; ++w) bits[w] = 0;
    for (uint32_t c = 0; c < n_cells; ++c)
        if (density[c] > threshold) { bits[c >> 5] |= 1u << (c & 31); ++set; }
    return set;
}

uint32_t dgo_march_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                            const uint32_t *seg_slot, uint32_t seg_begin, uint32_t seg_end, uint32_t k_max,
                            const float *aabb6, const dgo_occ *g, const uint32_t *bits, float dt,
                            uint32_t max_steps, uint64_t seed, uint32_t *first, float *u, float *delta,
                            float *t_samples, uint32_t *sample_ray)
{
    float inv_ext[3];
    for (int a = 0; a < 3; ++a) inv_ext[a] = 1.0f / (aabb6[3 + a] - aabb6[a]);
    uint32_t kept = 0;
    for (uint32_t j = seg_begin; j < seg_end; ++j) {
        first[j - seg_begin] = kept;
        uint32_t r = seg_ray[j], k = seg_slot[j];
        float t_in = seg_t[((uint64_t)r * k_max + k) * 2], t_out = seg_t[((uint64_t)r * k_max + k) * 2 + 1];
        float len = t_out - t_in;
        float wanted = ceilf(len / dt);                 /* strata no wider than the marching step */
        uint32_t n = wanted >= (float)max_steps ? max_steps : (wanted >= 1.0f ? (uint32_t)wanted : 1u);
        float width = len / (float)n;
        for (uint32_t s = 0; s < n; ++s) {
            float xi = dgo_jitter(seed, r, k, s);
            float t = t_in + ((float)s + xi) * width;
            float u3[3];
            for (int a = 0; a < 3; ++a) {
                float x = fmaf(t, d[3 * r + a], o[3 * r + a]);
                u3[a] = (x - aabb6[a]) * inv_ext[a];
            }
            uint32_t c = dgo_occ_cell(g, u3);
            if (!((bits[c >> 5] >> (c & 31)) & 1u)) continue;      /* empty space is skipped */
            if (u) {
                for (int a = 0; a < 3; ++a) u[3 * (uint64_t)kept + a] = u3[a];
                delta[kept] = width;
                t_samples[kept] = t;
                sample_ray[kept] = r;
            }
            ++kept;
        }
    }
    first[seg_end - seg_begin] = kept;
    return kept;
}

void dgo_composite_fwd_ragged(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                              const uint32_t *first, double *C, double *T)
{
    for (uint32_t j = 0; j < n_seg; ++j)
        dgo_composite_fwd(sigma + first[j], rgb + 3 * (uint64_t)first[j], delta + first[j], 1,
                          first[j + 1] - first[j], C + 3 * (uint64_t)j, T + j);
}

void dgo_composite_bwd_ragged(const double *sigma, const double *rgb, const double *delta, uint32_t n_seg,
                              const uint32_t *first, const double *gC, const double *gT, double *dsigma,
                              double *drgb)
{
    for (uint32_t j = 0; j < n_seg; ++j)
        dgo_composite_bwd(sigma + first[j], rgb + 3 * (uint64_t)first[j], delta + first[j], 1,
                          first[j + 1] - first[j], gC + 3 * (uint64_t)j, gT + j, dsigma + first[j],
                          drgb + 3 * (uint64_t)first[j]);
}

void dgo_composite_depth_ragged(const double *sigma, const double *delta, const double *t, uint32_t n_seg,
                                const uint32_t *first, double *D)
{
    for (uint32_t j = 0; j < n_seg; ++j)
        dgo_composite_depth(sigma + first[j], delta + first[j], t + first[j], 1, first[j + 1] - first[j], D + j);
}
