/* TEST INFRASTRUCTURE -- second, plain-C fp64 oracle of R-FAST's activation round.
 *
 * Only the tests and the benchmark's cpu_baseline leg load this file.  It shares
 * no code with the HIP library and none with the NumPy oracle next to it: it was
 * written separately from Algorithm 1 / Algorithm 2 of the paper, so that the two
 * oracles check each other, and so that the CPU baseline is a compiled program
 * (one thread, or OpenMP over the coordinates) rather than an interpreter.
 *
 * Scope: the separable objective f_i(x) = 1/2 sum_k h_ik (x_k - c_ik)^2 with
 * additive counter-based Gaussian gradient noise (the objective of the large
 * configurations), any pair of graphs (W row-stochastic, A column-stochastic,
 * CSR with row = receiver, diagonal included), any schedule.
 *
 * What one round does (every active node, all reading start-of-round state):
 *   resolve   on each in-edge (j -> i): u = t_j at the start of round r - delay;
 *             the newest version <= u that was delivered on this edge; the stamp
 *             kept is the larger of that and the stamp already held
 *   S1        v = x_i - gamma z_i
 *   S2a       x_i <- w_ii v + sum_{j != i} w_ij v_j[stamp]
 *   S2b       g' = grad f_i(x_i; zeta^{t_i+1});
 *             z_half = z_i + sum_{j != i} (rho_ij[stamp] - rho~_ij) + g' - g_i
 *   S2c       z_i <- a_ii z_half;  rho_li[t_i+1] = rho_li[t_i] + a_li z_half  (l != i)
 *   S3        v_i[t_i+1] = v; a version sent on an edge whose drop bit is set is never
 *             visible there, unless the burst-1 versions before it were all lost too
 *   S4        rho~_ij <- the rho_ij[stamp] consumed
 *   S5        t_i <- t_i + 1
 * Every version of v_i and rho_li ever published is kept in a growing array indexed
 * by the version number (nothing wraps around), freed once no reader may ask for it.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o librfast_oracle_c.so rfast_oracle_c.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int src, dst;       /* sender j, receiver i */
  double w;
  int64_t stamp;      /* largest stamp picked up so far */
  uint8_t* delivered; /* per version; grows */
  int64_t n_deliv;
} edge_t;

typedef struct {
  double** ver; /* ver[t] = published vector of version t (NULL once freed) */
  int64_t cap;
} history_t;

typedef struct rfo {
  int n, D, burst, d_max;
  int64_t p;
  int eR, eC;
  edge_t *R, *C;            /* off-diagonal entries in CSR order */
  int *r_ptr, *c_ptr;       /* [n+1] in-edges of node i are R[r_ptr[i] .. r_ptr[i+1]) */
  double *r_self, *c_self;  /* w_ii, a_ii */
  double *x, *z, *g;        /* [n][p] */
  double *h, *c;            /* objective */
  double noise_std;
  uint64_t noise_seed;
  int64_t* t;               /* local counters */
  history_t* v;             /* per node */
  history_t* rho;           /* per C edge (kept by the sender) */
  double* rho_tilde;        /* [eC][p] */
  int64_t** t_start;        /* t_start[s][j] = t_j at the start of round s */
  int64_t round_no, t_start_cap;
  double *v_new, *x_new, *g_new, *z_half; /* scratch of one activation */
} rfo;

/* ---------------------------------------------------------------- noise ---- */
/* Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0, k1). */
static void philox(uint32_t c[4], uint32_t k0, uint32_t k1) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    c[0] = n0; c[1] = (uint32_t)p1; c[2] = n2; c[3] = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

/* Standard normal of coordinate k for (node, version): coordinates come in groups of
 * four; words (o0, o1) give 4q, 4q+1 as r cos, r sin with u = ((o0 >> 8) + 1) / 2^24,
 * r = sqrt(-2 ln u), angle = 2 pi o1 / 2^32; (o2, o3) give 4q+2, 4q+3. */
static double normal_at(uint64_t seed, int node, int64_t version, int64_t k) {
  const uint64_t q = (uint64_t)k >> 2;
  uint32_t w[4] = {(uint32_t)q, (uint32_t)(q >> 32), (uint32_t)node, (uint32_t)version};
  philox(w, (uint32_t)seed, (uint32_t)(seed >> 32));
  const int pair = ((int)(k & 3)) >> 1;
  const double u = (double)((w[2 * pair] >> 8) + 1u) / 16777216.0;
  const double r = sqrt(-2.0 * log(u));
  const double angle = 6.283185307179586476925 * (double)w[2 * pair + 1] / 4294967296.0;
  return (k & 1) ? r * sin(angle) : r * cos(angle);
}

/* ------------------------------------------------------------- histories ---- */
static void hist_put(history_t* hs, int64_t t, double* vec) {
  if (t >= hs->cap) {
    int64_t cap = hs->cap ? hs->cap : 16;
    while (cap <= t) cap *= 2;
    hs->ver = (double**)realloc(hs->ver, (size_t)cap * sizeof(double*));
    for (int64_t q = hs->cap; q < cap; ++q) hs->ver[q] = NULL;
    hs->cap = cap;
  }
  hs->ver[t] = vec;
}
static void hist_free_before(history_t* hs, int64_t t) {
  for (int64_t q = t - 1; q >= 0 && q < hs->cap && hs->ver[q] != NULL; --q) {
    free(hs->ver[q]);
    hs->ver[q] = NULL;
  }
}
static void edge_set_delivered(edge_t* e, int64_t t, int yes) {
  if (t >= e->n_deliv) {
    int64_t cap = e->n_deliv ? e->n_deliv : 16;
    while (cap <= t) cap *= 2;
    e->delivered = (uint8_t*)realloc(e->delivered, (size_t)cap);
    memset(e->delivered + e->n_deliv, 0, (size_t)(cap - e->n_deliv));
    e->n_deliv = cap;
  }
  e->delivered[t] = (uint8_t)yes;
}

/* ------------------------------------------------------------ construction -- */
static void split(int n, const int32_t* rowptr, const int32_t* col, const double* w, int** ptr_out, edge_t** edges_out,
                  double** self_out, int* count_out) {
  int cnt = 0;
  for (int i = 0; i < n; ++i)
    for (int q = rowptr[i]; q < rowptr[i + 1]; ++q) cnt += col[q] != i;
  edge_t* ed = (edge_t*)calloc((size_t)(cnt > 0 ? cnt : 1), sizeof(edge_t));
  int* ptr = (int*)calloc((size_t)n + 1, sizeof(int));
  double* self = (double*)calloc((size_t)n, sizeof(double));
  int e = 0;
  for (int i = 0; i < n; ++i) {
    ptr[i] = e;
    for (int q = rowptr[i]; q < rowptr[i + 1]; ++q) {
      if (col[q] == i) {
        self[i] = w[q];
      } else {
        ed[e].src = col[q];
        ed[e].dst = i;
        ed[e].w = w[q];
        edge_set_delivered(&ed[e], 0, 1); /* version 0 (the zero vector) counts as delivered */
        ++e;
      }
    }
  }
  ptr[n] = e;
  *ptr_out = ptr; *edges_out = ed; *self_out = self; *count_out = cnt;
}

static void sample_gradient(const rfo* o, int i, const double* x, int64_t version, double* out) {
  const double* h = o->h + (size_t)i * o->p;
  const double* c = o->c + (size_t)i * o->p;
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < o->p; ++k) {
    double g = h[k] * (x[k] - c[k]);
    if (o->noise_std != 0.0) g += o->noise_std * normal_at(o->noise_seed, i, version, k);
    out[k] = g;
  }
}

rfo* rfo_create(int n, int64_t p, const int32_t* R_rowptr, const int32_t* R_col, const double* R_w,
                const int32_t* C_rowptr, const int32_t* C_col, const double* C_w, int D, int burst, const double* h,
                const double* c, double noise_std, uint64_t noise_seed, const double* x0) {
  rfo* o = (rfo*)calloc(1, sizeof(rfo));
  o->n = n; o->p = p; o->D = D; o->burst = burst; o->d_max = D - (burst - 1);
  o->noise_std = noise_std; o->noise_seed = noise_seed;
  split(n, R_rowptr, R_col, R_w, &o->r_ptr, &o->R, &o->r_self, &o->eR);
  split(n, C_rowptr, C_col, C_w, &o->c_ptr, &o->C, &o->c_self, &o->eC);
  const size_t np = (size_t)n * (size_t)p;
  o->x = (double*)calloc(np, sizeof(double));
  o->z = (double*)calloc(np, sizeof(double));
  o->g = (double*)calloc(np, sizeof(double));
  o->h = (double*)malloc(np * sizeof(double));
  o->c = (double*)malloc(np * sizeof(double));
  memcpy(o->h, h, np * sizeof(double));
  memcpy(o->c, c, np * sizeof(double));
  if (x0) memcpy(o->x, x0, np * sizeof(double));
  o->t = (int64_t*)calloc((size_t)n, sizeof(int64_t));
  o->v = (history_t*)calloc((size_t)n, sizeof(history_t));
  o->rho = (history_t*)calloc((size_t)(o->eC > 0 ? o->eC : 1), sizeof(history_t));
  o->rho_tilde = (double*)calloc((size_t)(o->eC > 0 ? o->eC : 1) * (size_t)p, sizeof(double));
  for (int i = 0; i < n; ++i) hist_put(&o->v[i], 0, (double*)calloc((size_t)p, sizeof(double)));
  for (int e = 0; e < o->eC; ++e) hist_put(&o->rho[e], 0, (double*)calloc((size_t)p, sizeof(double)));
  /* initialisation of Algorithm 1: z^0 = g^0 = sampled gradient at x^0 (sample version 0) */
  for (int i = 0; i < n; ++i) {
    sample_gradient(o, i, o->x + (size_t)i * p, 0, o->g + (size_t)i * p);
    memcpy(o->z + (size_t)i * p, o->g + (size_t)i * p, (size_t)p * sizeof(double));
  }
  o->t_start_cap = 64;
  o->t_start = (int64_t**)calloc((size_t)o->t_start_cap, sizeof(int64_t*));
  o->t_start[0] = (int64_t*)calloc((size_t)n, sizeof(int64_t));
  o->v_new = (double*)malloc((size_t)p * sizeof(double));
  o->x_new = (double*)malloc((size_t)p * sizeof(double));
  o->g_new = (double*)malloc((size_t)p * sizeof(double));
  o->z_half = (double*)malloc((size_t)p * sizeof(double));
  return o;
}

void rfo_destroy(rfo* o) {
  if (!o) return;
  for (int i = 0; i < o->n; ++i) {
    for (int64_t q = 0; q < o->v[i].cap; ++q) free(o->v[i].ver[q]);
    free(o->v[i].ver);
  }
  for (int e = 0; e < o->eC; ++e) {
    for (int64_t q = 0; q < o->rho[e].cap; ++q) free(o->rho[e].ver[q]);
    free(o->rho[e].ver);
    free(o->C[e].delivered);
  }
  for (int e = 0; e < o->eR; ++e) free(o->R[e].delivered);
  for (int64_t s = 0; s <= o->round_no; ++s) free(o->t_start[s]);
  free(o->t_start); free(o->v); free(o->rho); free(o->rho_tilde); free(o->R); free(o->C);
  free(o->r_ptr); free(o->c_ptr); free(o->r_self); free(o->c_self);
  free(o->x); free(o->z); free(o->g); free(o->h); free(o->c); free(o->t);
  free(o->v_new); free(o->x_new); free(o->g_new); free(o->z_half);
  free(o);
}

/* ------------------------------------------------------------------ round --- */
static int64_t newest_delivered_up_to(const edge_t* e, int64_t u) {
  for (int64_t t = u; t > 0; --t)
    if (t < e->n_deliv && e->delivered[t]) return t;
  return 0;
}

/* Is version t, whose packet on this edge was flagged lost, delivered anyway?  Yes when the
 * burst-1 versions before it were all lost on this edge (links do not fail forever). */
static int forced(const edge_t* e, int64_t t, int burst) {
  for (int k = 1; k < burst; ++k) {
    const int64_t q = t - k;
    if (q < 0 || (q < e->n_deliv && e->delivered[q])) return 0;
  }
  return 1;
}

static void activate(rfo* o, int i, const int64_t* stamp_R, const int64_t* stamp_C, double gamma, const uint8_t* drop_R,
                     const uint8_t* drop_C) {
  const int64_t p = o->p, t = o->t[i];
  double* x = o->x + (size_t)i * p;
  double* z = o->z + (size_t)i * p;
  double* g = o->g + (size_t)i * p;
  double *v_new = o->v_new, *x_new = o->x_new, *g_new = o->g_new, *z_half = o->z_half;
  /* S1 */
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < p; ++k) v_new[k] = x[k] - gamma * z[k];
  /* S2a */
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < p; ++k) x_new[k] = o->r_self[i] * v_new[k];
  for (int e = o->r_ptr[i]; e < o->r_ptr[i + 1]; ++e) {
    const double* vj = o->v[o->R[e].src].ver[stamp_R[e]];
    const double w = o->R[e].w;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < p; ++k) x_new[k] += w * vj[k];
  }
  /* S2b */
  sample_gradient(o, i, x_new, t + 1, g_new);
  memcpy(z_half, z, (size_t)p * sizeof(double));
  for (int e = o->c_ptr[i]; e < o->c_ptr[i + 1]; ++e) {
    const double* rho = o->rho[e].ver[stamp_C[e]];
    double* rt = o->rho_tilde + (size_t)e * p;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < p; ++k) {
      z_half[k] += rho[k] - rt[k];
      rt[k] = rho[k]; /* S4: buffer what was consumed */
    }
    o->C[e].stamp = stamp_C[e];
  }
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < p; ++k) z_half[k] += g_new[k] - g[k];
  /* S2c: keep a_ii, push a_li to every out-neighbour l as a running sum; S3: publish */
  for (int e = 0; e < o->eC; ++e) {
    if (o->C[e].src != i) continue;
    const double* cur = o->rho[e].ver[t];
    double* nxt = (double*)malloc((size_t)p * sizeof(double));
    const double a = o->C[e].w;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < p; ++k) nxt[k] = cur[k] + a * z_half[k];
    hist_put(&o->rho[e], t + 1, nxt);
    edge_set_delivered(&o->C[e], t + 1, !drop_C[e] || forced(&o->C[e], t + 1, o->burst));
    hist_free_before(&o->rho[e], t - o->D - 1);
  }
  for (int e = 0; e < o->eR; ++e) {
    if (o->R[e].src != i) continue;
    edge_set_delivered(&o->R[e], t + 1, !drop_R[e] || forced(&o->R[e], t + 1, o->burst));
  }
  for (int e = o->r_ptr[i]; e < o->r_ptr[i + 1]; ++e) o->R[e].stamp = stamp_R[e];
  double* pub = (double*)malloc((size_t)p * sizeof(double));
  memcpy(pub, v_new, (size_t)p * sizeof(double));
  hist_put(&o->v[i], t + 1, pub);
  hist_free_before(&o->v[i], t - o->D - 1);
  /* commit; S5 */
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < p; ++k) {
    x[k] = x_new[k];
    z[k] = o->c_self[i] * z_half[k];
    g[k] = g_new[k];
  }
  o->t[i] = t + 1;
}

/* returns 0, or -1 if a delay lies outside [0, d_max] */
int rfo_round(rfo* o, const uint8_t* active, const int32_t* delay_R, const int32_t* delay_C, const uint8_t* drop_R,
              const uint8_t* drop_C, double gamma) {
  for (int e = 0; e < o->eR; ++e)
    if (delay_R[e] < 0 || delay_R[e] > o->d_max) return -1;
  for (int e = 0; e < o->eC; ++e)
    if (delay_C[e] < 0 || delay_C[e] > o->d_max) return -1;
  const int64_t r = o->round_no;
  /* every active node resolves its stamps against the state at the start of the round */
  int64_t* stamp_R = (int64_t*)malloc((size_t)(o->eR > 0 ? o->eR : 1) * sizeof(int64_t));
  int64_t* stamp_C = (int64_t*)malloc((size_t)(o->eC > 0 ? o->eC : 1) * sizeof(int64_t));
  for (int e = 0; e < o->eR; ++e) {
    const int64_t seen_round = r - delay_R[e] > 0 ? r - delay_R[e] : 0;
    const int64_t cand = newest_delivered_up_to(&o->R[e], o->t_start[seen_round][o->R[e].src]);
    stamp_R[e] = cand > o->R[e].stamp ? cand : o->R[e].stamp;
  }
  for (int e = 0; e < o->eC; ++e) {
    const int64_t seen_round = r - delay_C[e] > 0 ? r - delay_C[e] : 0;
    const int64_t cand = newest_delivered_up_to(&o->C[e], o->t_start[seen_round][o->C[e].src]);
    stamp_C[e] = cand > o->C[e].stamp ? cand : o->C[e].stamp;
  }
  for (int i = 0; i < o->n; ++i)
    if (active[i]) activate(o, i, stamp_R, stamp_C, gamma, drop_R, drop_C);
  free(stamp_R);
  free(stamp_C);
  o->round_no = r + 1;
  if (o->round_no >= o->t_start_cap) {
    o->t_start_cap *= 2;
    o->t_start = (int64_t**)realloc(o->t_start, (size_t)o->t_start_cap * sizeof(int64_t*));
  }
  o->t_start[o->round_no] = (int64_t*)malloc((size_t)o->n * sizeof(int64_t));
  memcpy(o->t_start[o->round_no], o->t, (size_t)o->n * sizeof(int64_t));
  return 0;
}

/* ---------------------------------------------------------------- read-out -- */
void rfo_get_state(const rfo* o, double* x, double* z, double* g, int64_t* t, int64_t* stamp_R, int64_t* stamp_C) {
  const size_t np = (size_t)o->n * (size_t)o->p;
  if (x) memcpy(x, o->x, np * sizeof(double));
  if (z) memcpy(z, o->z, np * sizeof(double));
  if (g) memcpy(g, o->g, np * sizeof(double));
  if (t) memcpy(t, o->t, (size_t)o->n * sizeof(int64_t));
  if (stamp_R) for (int e = 0; e < o->eR; ++e) stamp_R[e] = o->R[e].stamp;
  if (stamp_C) for (int e = 0; e < o->eC; ++e) stamp_C[e] = o->C[e].stamp;
}

/* latest running sum and buffer of C edge e (Lemma 3 is checked from these by the caller) */
void rfo_get_edge(const rfo* o, int e, double* rho_latest, double* rho_tilde) {
  memcpy(rho_latest, o->rho[e].ver[o->t[o->C[e].src]], (size_t)o->p * sizeof(double));
  memcpy(rho_tilde, o->rho_tilde + (size_t)e * o->p, (size_t)o->p * sizeof(double));
}

int rfo_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void rfo_set_threads(int k) {
#ifdef _OPENMP
  omp_set_num_threads(k);
#else
  (void)k;
#endif
}
