/*
 * Seeded synthetic inputs: power-law graphs (COO edge lists) and vertex
 * feature matrices.  This file produces INPUTS only; it holds none of the
 * aggregation arithmetic and is used by both the CPU checker and the GPU
 * harness so that the two see the same bytes.
 *
 * The graphs take their vertex/edge counts and degree shape from the paper's
 * dataset table (Section III, Table II); the datasets themselves are not used.
 *
 * Randomness: one counter-based generator, a pure function of
 * (seed, stream, counter), so results do not depend on thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t fmix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t rnd_u64(uint64_t seed, uint64_t stream, uint64_t ctr) {
  uint64_t h = fmix64(seed + 0x9E3779B97F4A7C15ull * (stream + 1));
  return fmix64(h ^ fmix64(ctr + 0xD1B54A32D192ED03ull));
}

/* uniform in the open interval (0,1) */
static inline double rnd_u01(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return ((double)(rnd_u64(seed, stream, ctr) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

enum { STREAM_W = 1, STREAM_EDGE_A = 2, STREAM_EDGE_B = 3, STREAM_COVER = 4, STREAM_FEAT = 5 };

/* first index with cum[idx] > t (cum is non-decreasing, cum[n-1] = total) */
static inline int64_t pick(const double* cum, int64_t n, double t) {
  int64_t lo = 0, hi = n - 1;
  while (lo < hi) {
    int64_t mid = (lo + hi) >> 1;
    if (cum[mid] > t) hi = mid; else lo = mid + 1;
  }
  return lo;
}

typedef struct { uint64_t* slot; uint64_t mask; } pairset;

static int pairset_init(pairset* s, int64_t expect) {
  uint64_t cap = 1024;
  while (cap < (uint64_t)expect * 2 + 16) cap <<= 1;
  s->slot = (uint64_t*)calloc(cap, sizeof(uint64_t));
  s->mask = cap - 1;
  return s->slot ? 0 : -1;
}

/* returns 1 if newly inserted, 0 if already present */
static inline int pairset_add(pairset* s, int64_t u, int64_t v) {
  uint64_t a = (uint64_t)(u < v ? u : v), b = (uint64_t)(u < v ? v : u);
  uint64_t key = ((a << 32) | b) + 1; /* never 0 */
  uint64_t i = fmix64(key) & s->mask;
  for (;;) {
    uint64_t cur = s->slot[i];
    if (cur == 0) { s->slot[i] = key; return 1; }
    if (cur == key) return 0;
    i = (i + 1) & s->mask;
  }
}

static inline void pairset_prefetch(const pairset* s, int64_t u, int64_t v) {
  uint64_t a = (uint64_t)(u < v ? u : v), b = (uint64_t)(u < v ? v : u);
  uint64_t key = ((a << 32) | b) + 1;
  __builtin_prefetch(&s->slot[fmix64(key) & s->mask]);
}

/*
 * Undirected simple graph with M edges on N vertices, written as 2M directed
 * edges (slot 2k holds u->v, slot 2k+1 holds v->u).
 *
 * Each vertex gets a propensity w from a truncated Pareto law on [1,R] with
 * density ~ w^-alpha (inverse CDF).  Candidate pairs are drawn with both ends
 * proportional to w, in counter order; self pairs and pairs already present
 * are skipped; the first M accepted pairs are kept.  With cover_all != 0 every
 * vertex first receives one edge to a w-proportional partner.
 *
 * Returns the number of candidate draws consumed, or -1 on failure.
 */
int64_t synth_powerlaw_graph(int64_t N, int64_t M, double alpha, double R, uint64_t seed,
                             int cover_all, int32_t* src, int32_t* dst) {
  if (N < 2 || M < 0 || alpha <= 1.0 || R <= 1.0) return -1;
  if ((double)M > 0.45 * (double)N * (double)(N - 1)) return -1;
  double* cum = (double*)malloc(sizeof(double) * (size_t)N);
  if (!cum) return -1;
  const double tail = pow(R, 1.0 - alpha);
  double run = 0.0;
  for (int64_t v = 0; v < N; ++v) {
    double u = rnd_u01(seed, STREAM_W, (uint64_t)v);
    double w = pow(1.0 - u * (1.0 - tail), 1.0 / (1.0 - alpha));
    run += w;
    cum[v] = run;
  }
  const double total = run;
  pairset set;
  if (pairset_init(&set, M) != 0) { free(cum); return -1; }

  int64_t m = 0;
  if (cover_all) {
    uint64_t ctr = 0;
    for (int64_t v = 0; v < N && m < M; ++v) {
      for (;;) {
        int64_t p = pick(cum, N, rnd_u01(seed, STREAM_COVER, ctr++) * total);
        if (p == v) continue;
        if (!pairset_add(&set, v, p)) break; /* pair exists: v is already covered */
        src[2 * m] = (int32_t)v; dst[2 * m] = (int32_t)p;
        src[2 * m + 1] = (int32_t)p; dst[2 * m + 1] = (int32_t)v;
        ++m;
        break;
      }
    }
  }

  enum { BATCH = 1 << 20, AHEAD = 16 };
  int32_t* ca = (int32_t*)malloc(sizeof(int32_t) * BATCH);
  int32_t* cb = (int32_t*)malloc(sizeof(int32_t) * BATCH);
  if (!ca || !cb) { free(ca); free(cb); free(cum); free(set.slot); return -1; }
  uint64_t draws = 0;
  while (m < M) {
    /* draw a batch of candidates (any thread count gives the same values) */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < BATCH; ++i) {
      ca[i] = (int32_t)pick(cum, N, rnd_u01(seed, STREAM_EDGE_A, draws + (uint64_t)i) * total);
      cb[i] = (int32_t)pick(cum, N, rnd_u01(seed, STREAM_EDGE_B, draws + (uint64_t)i) * total);
    }
    int64_t i = 0;
    for (; i < BATCH && m < M; ++i) {
      if (i + AHEAD < BATCH) pairset_prefetch(&set, ca[i + AHEAD], cb[i + AHEAD]);
      int64_t u = ca[i], v = cb[i];
      if (u == v) continue;
      if (!pairset_add(&set, u, v)) continue;
      src[2 * m] = (int32_t)u; dst[2 * m] = (int32_t)v;
      src[2 * m + 1] = (int32_t)v; dst[2 * m + 1] = (int32_t)u;
      ++m;
    }
    draws += (uint64_t)i;
    if (draws > (uint64_t)M * 64 + (1u << 24)) { m = -1; break; } /* saturated */
  }
  free(ca); free(cb); free(cum); free(set.slot);
  return m < 0 ? -1 : (int64_t)draws;
}

/* standard normal by Box-Muller, element i of the stream keyed by seed */
static inline float normal_at(uint64_t seed, uint64_t i) {
  uint64_t k = i >> 1;
  double u1 = rnd_u01(seed, STREAM_FEAT, 2 * k);
  double u2 = rnd_u01(seed, STREAM_FEAT, 2 * k + 1);
  double r = sqrt(-2.0 * log(u1));
  double a = 6.283185307179586476925286766559 * u2;
  return (float)((i & 1) ? r * sin(a) : r * cos(a));
}

void synth_normal_f32(int64_t n, uint64_t seed, float mean, float std, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = mean + std * normal_at(seed, (uint64_t)i);
}

/* fp32 -> bf16 bits, round to nearest even; NaN stays NaN */
static inline uint16_t bf16_rne(float f) {
  uint32_t b;
  memcpy(&b, &f, 4);
  if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x40u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (uint16_t)(b >> 16);
}

void synth_normal_bf16(int64_t n, uint64_t seed, float mean, float std, uint16_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = bf16_rne(mean + std * normal_at(seed, (uint64_t)i));
}

void synth_f32_to_bf16(int64_t n, const float* in, uint16_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = bf16_rne(in[i]);
}

void synth_bernoulli_f32(int64_t n, double p, uint64_t seed, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = rnd_u01(seed, STREAM_FEAT, (uint64_t)i) < p ? 1.0f : 0.0f;
}

/* uniform integers in [0, hi) — for small directed test graphs */
void synth_randint_i32(int64_t n, int32_t hi, uint64_t seed, uint64_t stream, int32_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = (int32_t)(rnd_u64(seed, 16 + stream, (uint64_t)i) % (uint64_t)hi);
}
