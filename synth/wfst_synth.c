/*
 * Seeded synthetic inputs for WFST decoding: decoding graphs in CSR form and rows of
 * acoustic log-likelihoods.
 *
 * This module only draws numbers.  It contains none of the decoder's arithmetic and is
 * shared by the CPU checker and by the GPU library's tests and benchmark so that both
 * sides decode byte-identical inputs.
 *
 * Every value is a pure function of (seed, stream, index) through a 64-bit integer
 * mixing function, so any slice can be produced anywhere, in any order, with the same
 * bytes.  The log-likelihood recipe uses integer arithmetic up to one multiply and one
 * or two adds in fp32, each individually rounded (build with -ffp-contract=off); the
 * device generator in loglikes.hip repeats exactly these steps.
 *
 * The inputs stand in for the decoding graphs and acoustic-model posteriors of the
 * paper's experiments (Section 4), which are not available: state/arc counts, degree
 * skew, fraction of non-emitting arcs, number of pdfs and value ranges follow the
 * workload descriptions used by this repository's configurations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
  z ^= z >> 27; z *= 0x94D049BB133111EBULL;
  z ^= z >> 31;
  return z;
}

/* hash of a (seed, a, b) triple; distinct tags/indices give decorrelated outputs */
static inline uint64_t h3(uint64_t seed, uint64_t a, uint64_t b) {
  uint64_t z = mix64(seed + GOLDEN);
  z = mix64(z ^ (a * 0xD1342543DE82EF95ULL + 0x632BE59BD9B4E019ULL));
  return mix64(z + b * GOLDEN);
}

/* uniform double in [0,1) with 53 bits */
static inline double u01(uint64_t h) { return (double)(h >> 11) * (1.0 / 9007199254740992.0); }

enum { TAG_DEG = 1, TAG_ZERO = 2, TAG_DST = 3, TAG_PDF = 4, TAG_W = 5, TAG_OL = 6,
       TAG_EPS_SRC = 7, TAG_EPS_DST = 8, TAG_EPS_W = 9, TAG_EPS_OL = 10, TAG_FINAL = 11,
       TAG_FINAL_W = 12, TAG_ADJ = 13, TAG_LEN = 14, TAG_LL = 15, TAG_TRUE = 16 };

typedef struct {
  uint64_t seed;
  int32_t  num_states;
  int64_t  num_emit;      /* exact number of emitting arcs; 0 = whatever the degree model draws */
  int64_t  num_eps;       /* exact number of non-emitting arcs (all go to higher state ids)      */
  int32_t  degree_model;  /* 0 fixed(deg_param), 1 geometric(mean deg_param, k>=1), 2 power law  */
  double   deg_param;     /* fixed degree / geometric mean / power-law exponent                  */
  int32_t  deg_max;       /* cap on the emitting out-degree                                      */
  int32_t  num_pdfs;
  int32_t  vocab;         /* olabels are drawn from [1, vocab] on 10% of the arcs, else 0        */
  float    weight_max;    /* arc weights uniform in [0, weight_max)                              */
  int32_t  num_final;     /* exact number of final states                                        */
  float    final_max;     /* final costs uniform in [0, final_max)                               */
  int32_t  interleave;    /* 0: emitting arcs first within a state; 1: epsilon arcs first        */
} synth_graph_spec;

/* Draw the emitting out-degree of every state and force the requested total. */
static int draw_degrees(const synth_graph_spec *sp, int32_t *deg, int64_t *total_out) {
  const int32_t Q = sp->num_states;
  const int32_t dmax = sp->deg_max > 0 ? sp->deg_max : 1;
  double *cdf = NULL;
  double p_one = 0.0;
  if (sp->degree_model == 2) {
    cdf = (double *)malloc(sizeof(double) * (size_t)dmax);
    if (!cdf) return -1;
    double z = 0.0, m = 0.0;
    for (int k = 1; k <= dmax; ++k) { double p = pow((double)k, -sp->deg_param); z += p; m += p * k; }
    double acc = 0.0;
    for (int k = 1; k <= dmax; ++k) { acc += pow((double)k, -sp->deg_param) / z; cdf[k - 1] = acc; }
    double mean = m / z;
    if (sp->num_emit > 0) {
      double want = (double)sp->num_emit / (double)Q;
      /* the pure power law has a larger mean than asked for: mix in states with exactly one
         emitting arc (never zero: like a real decoding graph, every state can move on) */
      if (want < mean && mean > 1.0) p_one = (mean - want) / (mean - 1.0);
    }
  }
  int64_t total = 0;
  for (int32_t s = 0; s < Q; ++s) {
    int32_t d;
    if (sp->degree_model == 0) {
      d = (int32_t)sp->deg_param;
    } else if (sp->degree_model == 1) {
      double q = 1.0 - 1.0 / sp->deg_param;
      double u = 1.0 - u01(h3(sp->seed, TAG_DEG, (uint64_t)s));      /* (0,1] */
      d = 1 + (int32_t)floor(log(u) / log(q));
    } else {
      if (u01(h3(sp->seed, TAG_ZERO, (uint64_t)s)) < p_one) {
        d = 1;
      } else {
        double u = u01(h3(sp->seed, TAG_DEG, (uint64_t)s));
        int lo = 0, hi = dmax - 1;                                    /* first k with cdf >= u */
        while (lo < hi) { int mid = (lo + hi) >> 1; if (cdf[mid] >= u) hi = mid; else lo = mid + 1; }
        d = lo + 1;
      }
    }
    if (d > dmax) d = dmax;
    if (d < 0) d = 0;
    deg[s] = d;
    total += d;
  }
  free(cdf);
  /* the start state must be able to move; in the skewed model, where most states have a
     single successor and some none, it fans out widely like the start of a real decoding
     graph, otherwise most streams would die within a few frames */
  int32_t d0 = 1;
  if (sp->degree_model == 2) d0 = dmax < 256 ? dmax : 256;
  if (deg[0] < d0) { total += d0 - deg[0]; deg[0] = d0; }
  if (sp->num_emit > 0) {
    /* walk states in a hashed order, nudging degrees by one until the total is exact */
    uint64_t i = 0;
    while (total != sp->num_emit) {
      int32_t s = (int32_t)(h3(sp->seed, TAG_ADJ, i++) % (uint64_t)Q);
      if (total > sp->num_emit) { if (s != 0 && deg[s] > 1) { deg[s]--; total--; } }
      else if (deg[s] < dmax) { deg[s]++; total++; }
      if (i > (uint64_t)Q * 4096ULL) return -2;                       /* cannot reach the total */
    }
  }
  *total_out = total;
  return 0;
}

/* Number of arcs the graph will have (emitting + epsilon); needed to size the arrays. */
int synth_graph_num_arcs(const synth_graph_spec *sp, int64_t *num_emit, int64_t *num_arcs) {
  if (!sp || sp->num_states < 2) return -1;
  int32_t *deg = (int32_t *)malloc(sizeof(int32_t) * (size_t)sp->num_states);
  if (!deg) return -1;
  int64_t total = 0;
  int rc = draw_degrees(sp, deg, &total);
  free(deg);
  if (rc) return rc;
  *num_emit = total;
  *num_arcs = total + sp->num_eps;
  return 0;
}

/*
 * Fill caller-allocated CSR arrays.  row_offsets has num_states+1 entries, the per-arc
 * arrays have num_arcs entries (from synth_graph_num_arcs), final_cost has num_states.
 */
int synth_graph_fill(const synth_graph_spec *sp, int64_t *row_offsets, int32_t *ilabel,
                     int32_t *olabel, float *weight, int32_t *nextstate, float *final_cost) {
  if (!sp || sp->num_states < 2) return -1;
  const int32_t Q = sp->num_states;
  int32_t *deg = (int32_t *)malloc(sizeof(int32_t) * (size_t)Q);
  int32_t *neps = (int32_t *)calloc((size_t)Q, sizeof(int32_t));
  if (!deg || !neps) { free(deg); free(neps); return -1; }
  int64_t n_emit = 0;
  int rc = draw_degrees(sp, deg, &n_emit);
  if (rc) { free(deg); free(neps); return rc; }
  /* epsilon arcs: source uniform over states that have a successor id */
  for (int64_t i = 0; i < sp->num_eps; ++i) {
    int32_t s = (int32_t)(h3(sp->seed, TAG_EPS_SRC, (uint64_t)i) % (uint64_t)(Q - 1));
    neps[s]++;
  }
  row_offsets[0] = 0;
  for (int32_t s = 0; s < Q; ++s) row_offsets[s + 1] = row_offsets[s] + deg[s] + neps[s];
  /* emitting arcs */
  int64_t e = 0;                                   /* running emitting-arc ordinal */
  for (int32_t s = 0; s < Q; ++s) {
    int64_t base = row_offsets[s] + (sp->interleave ? neps[s] : 0);
    for (int32_t k = 0; k < deg[s]; ++k, ++e) {
      int64_t a = base + k;
      nextstate[a] = (int32_t)(h3(sp->seed, TAG_DST, (uint64_t)e) % (uint64_t)Q);
      ilabel[a] = 1 + (int32_t)(h3(sp->seed, TAG_PDF, (uint64_t)e) % (uint64_t)sp->num_pdfs);
      weight[a] = (float)(h3(sp->seed, TAG_W, (uint64_t)e) >> 40) * (1.0f / 16777216.0f) * sp->weight_max;
      uint64_t ho = h3(sp->seed, TAG_OL, (uint64_t)e);
      olabel[a] = (ho % 10u == 0) ? 1 + (int32_t)((ho >> 8) % (uint64_t)sp->vocab) : 0;
    }
  }
  /* epsilon arcs, appended per source state in draw order */
  int32_t *fillp = (int32_t *)calloc((size_t)Q, sizeof(int32_t));
  if (!fillp) { free(deg); free(neps); return -1; }
  for (int64_t i = 0; i < sp->num_eps; ++i) {
    int32_t s = (int32_t)(h3(sp->seed, TAG_EPS_SRC, (uint64_t)i) % (uint64_t)(Q - 1));
    int64_t a = row_offsets[s] + (sp->interleave ? 0 : deg[s]) + fillp[s]++;
    nextstate[a] = s + 1 + (int32_t)(h3(sp->seed, TAG_EPS_DST, (uint64_t)i) % (uint64_t)(Q - 1 - s));
    ilabel[a] = 0;
    weight[a] = (float)(h3(sp->seed, TAG_EPS_W, (uint64_t)i) >> 40) * (1.0f / 16777216.0f) * sp->weight_max;
    uint64_t ho = h3(sp->seed, TAG_EPS_OL, (uint64_t)i);
    olabel[a] = (ho % 10u == 0) ? 1 + (int32_t)((ho >> 8) % (uint64_t)sp->vocab) : 0;
  }
  free(fillp);
  /* final states: exactly num_final distinct states */
  for (int32_t s = 0; s < Q; ++s) final_cost[s] = INFINITY;
  int32_t placed = 0;
  for (uint64_t i = 0; placed < sp->num_final && placed < Q; ++i) {
    int32_t s = (int32_t)(h3(sp->seed, TAG_FINAL, i) % (uint64_t)Q);
    if (isinf(final_cost[s])) {
      final_cost[s] = (float)(h3(sp->seed, TAG_FINAL_W, i) >> 40) * (1.0f / 16777216.0f) * sp->final_max;
      placed++;
    }
  }
  free(deg); free(neps);
  return 0;
}

/* Length of stream `stream`: uniform integer in [lo, hi]. */
int32_t synth_stream_length(uint64_t seed, int32_t stream, int32_t lo, int32_t hi) {
  if (hi <= lo) return lo;
  return lo + (int32_t)(h3(seed, TAG_LEN, (uint64_t)stream) % (uint64_t)(hi - lo + 1));
}

/* Index of the boosted ("true") pdf of one frame. */
int32_t synth_true_pdf(uint64_t seed, int32_t stream, int32_t frame, int32_t num_pdfs) {
  return (int32_t)(h3(seed ^ 0x5DEECE66DULL, TAG_TRUE + ((uint64_t)stream << 8), (uint64_t)frame) % (uint64_t)num_pdfs);
}

/*
 * One log-likelihood value.  z is the sum of twelve 16-bit uniforms, centred and scaled:
 * mean 0, variance 1, support (-6, 6) — an all-integer stand-in for a standard normal.
 * value = mu + sigma*z, plus `boost` on the frame's true pdf; every fp32 operation is
 * rounded on its own.
 */
static inline float ll_value(uint64_t base, int32_t p, float mu, float sigma) {
  uint64_t st = base + (uint64_t)(3 * (int64_t)p) * GOLDEN;
  int32_t sum = 0;
  for (int k = 0; k < 3; ++k) {
    uint64_t r = mix64(st + (uint64_t)k * GOLDEN);
    sum += (int32_t)(r & 0xFFFF) + (int32_t)((r >> 16) & 0xFFFF) + (int32_t)((r >> 32) & 0xFFFF) + (int32_t)(r >> 48);
  }
  float z = (float)(2 * sum - 12 * 65535) * (1.0f / 131072.0f);      /* exact in fp32 */
  float sz = sigma * z;
  return mu + sz;
}

/*
 * Fill rows [frame0, frame0+n_frames) of stream `stream` into out[n_frames][stride].
 * Columns >= num_pdfs (padding when stride > num_pdfs) are left untouched.
 */
int synth_loglikes_fill(uint64_t seed, int32_t stream, int32_t frame0, int32_t n_frames,
                        int32_t num_pdfs, float mu, float sigma, float boost,
                        float *out, int64_t stride) {
  if (!out || num_pdfs < 1 || stride < num_pdfs) return -1;
  for (int32_t f = 0; f < n_frames; ++f) {
    int32_t frame = frame0 + f;
    uint64_t base = h3(seed, TAG_LL + ((uint64_t)stream << 8), (uint64_t)frame);
    float *row = out + (int64_t)f * stride;
    for (int32_t p = 0; p < num_pdfs; ++p) row[p] = ll_value(base, p, mu, sigma);
    int32_t tp = synth_true_pdf(seed, stream, frame, num_pdfs);
    float v = row[tp];
    row[tp] = v + boost;
  }
  return 0;
}
