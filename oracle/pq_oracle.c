/*
 * pq_oracle.c -- plain fp64 CPU oracle for the PolarQuant hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * reference that the HIP library is checked against.  It shares no code,
 * header, table or constant with the GPU path; only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.
 *
 * Everything is double precision, uses libm atan2/cos/sin/sqrt/hypot, and
 * follows the paper's steps in the paper's order and notation:
 *   r^(l)      radii after level l            (Algorithm 1, procedure Polar)
 *   psi^(l)    angles of level l              (Definition 1)
 *   theta^(l)  codebook centroids of level l  (Eq. 3)
 *   J^(l)      quantised angle indices        (Algorithm 1, procedure Quant)
 * The practical configuration of Section 4.1 is the one encoded into
 * records: d = 128, L = 4 levels, 4 bits at level 1 and 2 bits at levels
 * 2..4, one 16-bit float radius per block of 16 coordinates.
 *
 * Parity status of each function is stated in its comment; functions whose
 * result no independent fact pins say "parity unpinned".
 *
 * OpenMP pragmas parallelise over independent vectors / cached rows only;
 * no blocking, fusion or reordering beyond the definitions.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_D 128            /* head dimension of Section 4.1's example   */
#define ORC_L 4              /* recursion depth L = 4 (Section 4.1)       */
#define ORC_BLOCK 16         /* 2^L coordinates share one stored radius   */
#define ORC_F16_MAX 65504.0  /* largest finite binary16: stored radii saturate there */
#define ORC_NBLK (ORC_D / ORC_BLOCK)
#define ORC_REC 62           /* 46 code bytes + 8 half radii per vector   */
#define ORC_NANG 120         /* 64 + 32 + 16 + 8 angles per vector        */

static const double ORC_PI = 3.14159265358979323846264338327950288;

/* ------------------------------------------------------------------ */
/* Random numbers the method draws: the Gaussian matrix behind S.      */
/* Counter-based: splitmix64 finaliser + Box-Muller, entry (i,j) uses  */
/* counter c = i*d + j.  The GPU library implements the same published */
/* generator on its own; nothing is shared.                            */
/* ------------------------------------------------------------------ */
static uint64_t orc_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static double orc_unit_open(uint64_t seed, uint64_t counter)
{
    uint64_t w = orc_mix64(orc_mix64(seed) + (counter + 1) * 0x9E3779B97F4A7C15ULL);
    return ((double)(w >> 11) + 0.5) * (1.0 / 9007199254740992.0); /* (0,1) */
}

/* G[i*d+j] ~ N(0,1), deterministic in (seed, i, j). */
void orc_gaussian_matrix(uint64_t seed, int d, double *G)
{
    for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j) {
            uint64_t c = (uint64_t)i * (uint64_t)d + (uint64_t)j;
            double u1 = orc_unit_open(seed, 2 * c);
            double u2 = orc_unit_open(seed, 2 * c + 1);
            G[i * d + j] = sqrt(-2.0 * log(u1)) * cos(2.0 * ORC_PI * u2);
        }
}

/* ------------------------------------------------------------------ */
/* Preconditioner S: a random rotation (Section 3.2 footnote, Section  */
/* 4.1): QR factorisation of a Gaussian matrix by Householder          */
/* reflections, S = Q * diag(sign(R_ii)) so that the factorisation is  */
/* the unique one with a positive diagonal of R.  Row-major d x d.     */
/* Pinned by: orthogonality, |det| = 1, agreement with LAPACK's QR.    */
/* ------------------------------------------------------------------ */
int orc_rotation_from_gaussian(const double *G, int d, double *S)
{
    double *R = (double *)malloc(sizeof(double) * d * d);
    double *Q = (double *)malloc(sizeof(double) * d * d);
    double *v = (double *)malloc(sizeof(double) * d);
    if (!R || !Q || !v) { free(R); free(Q); free(v); return -1; }
    memcpy(R, G, sizeof(double) * d * d);
    for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j) Q[i * d + j] = (i == j) ? 1.0 : 0.0;

    for (int k = 0; k < d; ++k) {
        /* Householder vector for column k of R, rows k..d-1 */
        double norm = 0.0;
        for (int i = k; i < d; ++i) norm += R[i * d + k] * R[i * d + k];
        norm = sqrt(norm);
        if (norm == 0.0) continue;
        double alpha = (R[k * d + k] > 0.0) ? -norm : norm;
        double vnorm2 = 0.0;
        for (int i = 0; i < d; ++i) v[i] = 0.0;
        for (int i = k; i < d; ++i) v[i] = R[i * d + k];
        v[k] -= alpha;
        for (int i = k; i < d; ++i) vnorm2 += v[i] * v[i];
        if (vnorm2 == 0.0) continue;
        /* R <- (I - 2 v v^T / v^T v) R */
        for (int j = 0; j < d; ++j) {
            double s = 0.0;
            for (int i = k; i < d; ++i) s += v[i] * R[i * d + j];
            s = 2.0 * s / vnorm2;
            for (int i = k; i < d; ++i) R[i * d + j] -= s * v[i];
        }
        /* Q <- Q (I - 2 v v^T / v^T v) */
        for (int i = 0; i < d; ++i) {
            double s = 0.0;
            for (int j = k; j < d; ++j) s += Q[i * d + j] * v[j];
            s = 2.0 * s / vnorm2;
            for (int j = k; j < d; ++j) Q[i * d + j] -= s * v[j];
        }
    }
    for (int j = 0; j < d; ++j) {
        double sgn = (R[j * d + j] < 0.0) ? -1.0 : 1.0;
        for (int i = 0; i < d; ++i) S[i * d + j] = Q[i * d + j] * sgn;
    }
    free(R); free(Q); free(v);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Angle density of level l >= 2 (Lemma 2):                            */
/*   f_l(psi) = Gamma(2^(l-1)) / (2^(2^(l-1)-2) Gamma(2^(l-2))^2)      */
/*              * sin^(2^(l-1)-1)(2 psi),   0 <= psi <= pi/2.          */
/* Pinned by: integrates to 1, symmetric about pi/4, empirical angle   */
/* histograms of Gaussian vectors (regularised incomplete beta CDF).   */
/* ------------------------------------------------------------------ */
double orc_angle_pdf(int level, double psi)
{
    if (level < 2) return 1.0 / (2.0 * ORC_PI);      /* uniform on [0,2pi) */
    double n = ldexp(1.0, level - 1);                 /* 2^(l-1) */
    double h = ldexp(1.0, level - 2);                 /* 2^(l-2) */
    double lognorm = lgamma(n) - (n - 2.0) * log(2.0) - 2.0 * lgamma(h);
    double s = sin(2.0 * psi);
    if (s <= 0.0) return (n - 1.0 == 0.0) ? exp(lognorm) : 0.0;
    return exp(lognorm + (n - 1.0) * log(s));
}

/* composite Simpson on [a,b] of psi^p * f_l(psi), p in {0,1,2} */
static double orc_moment(int level, double a, double b, int p, double shift)
{
    const int N = 4096;                               /* even */
    double h = (b - a) / N, acc = 0.0;
    for (int i = 0; i <= N; ++i) {
        double x = a + h * i;
        double w = (i == 0 || i == N) ? 1.0 : ((i & 1) ? 4.0 : 2.0);
        double g = orc_angle_pdf(level, x);
        double t = x - shift;
        acc += w * g * (p == 0 ? 1.0 : (p == 1 ? t : t * t));
    }
    return acc * h / 3.0;
}

/* ------------------------------------------------------------------ */
/* Codebook of one level (Algorithm 1 line 3, Eq. 3): the minimiser of */
/* the expected squared angle error under the level's density, i.e.    */
/* the continuous 1-D k-means fixed point (Lloyd-Max): boundaries are  */
/* midpoints of neighbouring centroids, centroids are conditional      */
/* means of their interval.  Level 1 is uniform on [0, 2 pi): its      */
/* optimum is the mid-points of K equal intervals.                     */
/*   centroids[K], boundaries[K+1] (boundaries[0] = lower end of the   */
/*   range, boundaries[K] = upper end).                                */
/* Pinned by: symmetry, centroid/midpoint conditions re-checked with   */
/* an independent quadrature, distortion not improvable by nudging.    */
/* ------------------------------------------------------------------ */
int orc_codebook(int level, int K, double *centroids, double *boundaries)
{
    if (K < 1) return -1;
    if (level == 1) {
        for (int k = 0; k <= K; ++k) boundaries[k] = 2.0 * ORC_PI * k / K;
        for (int k = 0; k < K; ++k) centroids[k] = 2.0 * ORC_PI * (k + 0.5) / K;
        return 0;
    }
    double lo = 0.0, hi = ORC_PI / 2.0;
    for (int k = 0; k < K; ++k) centroids[k] = lo + (hi - lo) * (k + 0.5) / K;
    for (int it = 0; it < 100000; ++it) {
        boundaries[0] = lo; boundaries[K] = hi;
        for (int k = 1; k < K; ++k) boundaries[k] = 0.5 * (centroids[k - 1] + centroids[k]);
        double delta = 0.0;
        for (int k = 0; k < K; ++k) {
            double m0 = orc_moment(level, boundaries[k], boundaries[k + 1], 0, 0.0);
            double m1 = orc_moment(level, boundaries[k], boundaries[k + 1], 1, 0.0);
            double c = m1 / m0;
            double dlt = fabs(c - centroids[k]);
            if (dlt > delta) delta = dlt;
            centroids[k] = c;
        }
        /* the fixed point is reached when the centroids stop moving; with more cells rounding in the
           quadrature keeps successive iterates a few 1e-16 apart, which is as converged as it gets */
        if (delta < 1e-15 || (it > 500 && delta < 1e-13)) break;
    }
    boundaries[0] = lo; boundaries[K] = hi;
    for (int k = 1; k < K; ++k) boundaries[k] = 0.5 * (centroids[k - 1] + centroids[k]);
    return 0;
}

/* Expected squared quantisation error of a codebook under f_l (Eq. 3). */
double orc_codebook_distortion(int level, int K, const double *centroids)
{
    double lo = 0.0, hi = (level == 1) ? 2.0 * ORC_PI : ORC_PI / 2.0, acc = 0.0;
    for (int k = 0; k < K; ++k) {
        double a = (k == 0) ? lo : 0.5 * (centroids[k - 1] + centroids[k]);
        double b = (k == K - 1) ? hi : 0.5 * (centroids[k] + centroids[k + 1]);
        acc += orc_moment(level, a, b, 2, centroids[k]);
    }
    return acc;
}

/* ------------------------------------------------------------------ */
/* Procedure Polar (Algorithm 1; Definition 1), general d = 2^p and    */
/* depth L <= p.  Input y[d].  Output psi holds the levels one after   */
/* another: d/2 angles of level 1, d/4 of level 2, ...; r holds the    */
/* d/2^L radii r^(L).  Level-1 angles lie in [0, 2 pi) (atan2 shifted  */
/* by 2 pi when negative), deeper levels in [0, pi/2].                 */
/* Pinned by: exact inverse, r^(L) = block norms, d = 2 textbook case. */
/* ------------------------------------------------------------------ */
void orc_polar(const double *y, int d, int L, double *psi, double *r)
{
    double *cur = (double *)malloc(sizeof(double) * d);
    memcpy(cur, y, sizeof(double) * d);                /* r^(0) = y */
    int n = d, off = 0;
    for (int l = 1; l <= L; ++l) {
        int half = n / 2;
        for (int j = 0; j < half; ++j) {
            double a = cur[2 * j], b = cur[2 * j + 1];
            double ang = atan2(b, a);                  /* tan^-1(r_2j / r_2j-1) */
            /* a tiny negative angle plus 2 pi may round to 2 pi itself; it is
               kept (its nearest centroid is the last one, as for the exact
               value just below 2 pi) */
            if (l == 1 && ang < 0.0) ang += 2.0 * ORC_PI;
            psi[off + j] = ang;
            cur[j] = hypot(a, b);                      /* in-place is safe: j <= 2j */
        }
        off += half;
        n = half;
    }
    memcpy(r, cur, sizeof(double) * n);
    free(cur);
}

/* Inverse of Polar (DeQuant's loop of Algorithm 1 with exact angles). */
void orc_polar_inverse(const double *psi, const double *r, int d, int L, double *y)
{
    double *cur = (double *)malloc(sizeof(double) * d);
    double *nxt = (double *)malloc(sizeof(double) * d);
    int n = d >> L;
    memcpy(cur, r, sizeof(double) * n);
    /* offset of level l inside psi */
    for (int l = L; l >= 1; --l) {
        int off = 0;
        for (int m = 1; m < l; ++m) off += d >> m;
        for (int j = 0; j < n; ++j) {
            nxt[2 * j]     = cur[j] * cos(psi[off + j]);
            nxt[2 * j + 1] = cur[j] * sin(psi[off + j]);
        }
        n *= 2;
        memcpy(cur, nxt, sizeof(double) * n);
    }
    memcpy(y, cur, sizeof(double) * d);
    free(cur); free(nxt);
}

/* Procedure Quant: index of the nearest centroid, |theta_k - psi|      */
/* linear (not circular) as written; lowest index wins a tie.           */
int orc_quant(double psi, const double *theta, int K)
{
    int best = 0;
    double bd = fabs(theta[0] - psi);
    for (int k = 1; k < K; ++k) {
        double dk = fabs(theta[k] - psi);
        if (dk < bd) { bd = dk; best = k; }
    }
    return best;
}

/* ------------------------------------------------------------------ */
/* IEEE binary16 <-> double, round-to-nearest-even, subnormals kept.   */
/* Pinned against numpy's float16 casts.                               */
/* ------------------------------------------------------------------ */
uint16_t orc_f64_to_f16(double x)
{
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs(x);
    if (isnan(a)) return (uint16_t)(sign | 0x7E00u);
    if (a == 0.0) return sign;
    if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);       /* rounds to inf */
    if (a < ldexp(1.0, -14)) {                                  /* subnormal range */
        double q = rint(ldexp(a, 24));                          /* ties to even */
        return (uint16_t)(sign | (uint16_t)q);                  /* 1024 -> smallest normal */
    }
    int e;
    double f = frexp(a, &e);                                    /* a = f 2^e, f in [0.5,1) */
    int E = e - 1;                                              /* a = (2f) 2^E */
    double m = rint(ldexp(f, 11));                              /* in [1024, 2048] */
    if (m >= 2048.0) { m = 1024.0; E += 1; }
    if (E > 15) return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | (uint16_t)((E + 15) << 10) | (uint16_t)((int)m - 1024));
}

double orc_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp(1024.0 + m, e - 25);
    return sign ? -v : v;
}

/* ------------------------------------------------------------------ */
/* Codebooks of the Section 4.1 configuration in one struct-free blob: */
/*   cb[0..15]  level-1 centroids (16), cb[16..19] level 2,            */
/*   cb[20..23] level 3, cb[24..27] level 4.                           */
/* ------------------------------------------------------------------ */
#define ORC_CB_LEN 28
static const int orc_cb_off[5] = {0, 0, 16, 20, 24};
static const int orc_cb_K[5]   = {0, 16, 4, 4, 4};

int orc_default_codebooks(double *cb)
{
    double bnd[17];
    for (int l = 1; l <= ORC_L; ++l)
        if (orc_codebook(l, orc_cb_K[l], cb + orc_cb_off[l], bnd)) return -1;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Canonical record of one d=128 vector (62 bytes).  The paper fixes   */
/* only "indices packed into 8-bit units" and the bit budget; this     */
/* order is this project's documented reading:                         */
/*   bytes  0..31  level 1: 64 codes in coordinate order, two per byte */
/*                 earlier code in the high nibble                     */
/*   bytes 32..39  level 2: 32 codes, four per byte, earlier = higher  */
/*   bytes 40..43  level 3: 16 codes, four per byte, earlier = higher  */
/*   bytes 44..45  level 4:  8 codes (code j = block j), same order    */
/*   bytes 46..61  8 binary16 radii, little endian, block order        */
/* ------------------------------------------------------------------ */
static void orc_pack_record(const int *J /*120 codes, level-major*/, const uint16_t *rad, uint8_t *rec)
{
    memset(rec, 0, ORC_REC);
    for (int j = 0; j < 64; ++j)
        rec[j / 2] |= (uint8_t)((J[j] & 15) << ((j & 1) ? 0 : 4));
    const int base[3] = {32, 40, 44}, cnt[3] = {32, 16, 8}, off[3] = {64, 96, 112};
    for (int t = 0; t < 3; ++t)
        for (int j = 0; j < cnt[t]; ++j)
            rec[base[t] + j / 4] |= (uint8_t)((J[off[t] + j] & 3) << (6 - 2 * (j & 3)));
    for (int b = 0; b < ORC_NBLK; ++b) {
        rec[46 + 2 * b] = (uint8_t)(rad[b] & 0xFF);
        rec[47 + 2 * b] = (uint8_t)(rad[b] >> 8);
    }
}

static void orc_unpack_record(const uint8_t *rec, int *J, uint16_t *rad)
{
    for (int j = 0; j < 64; ++j)
        J[j] = (rec[j / 2] >> ((j & 1) ? 0 : 4)) & 15;
    const int base[3] = {32, 40, 44}, cnt[3] = {32, 16, 8}, off[3] = {64, 96, 112};
    for (int t = 0; t < 3; ++t)
        for (int j = 0; j < cnt[t]; ++j)
            J[off[t] + j] = (rec[base[t] + j / 4] >> (6 - 2 * (j & 3))) & 3;
    for (int b = 0; b < ORC_NBLK; ++b)
        rad[b] = (uint16_t)(rec[46 + 2 * b] | (rec[47 + 2 * b] << 8));
}

void orc_pack(const int32_t *J, const uint16_t *rad, int64_t n, uint8_t *rec)
{
    for (int64_t i = 0; i < n; ++i) {
        int tmp[ORC_NANG];
        for (int a = 0; a < ORC_NANG; ++a) tmp[a] = J[i * ORC_NANG + a];
        orc_pack_record(tmp, rad + i * ORC_NBLK, rec + i * ORC_REC);
    }
}

void orc_unpack(const uint8_t *rec, int64_t n, int32_t *J, uint16_t *rad)
{
    for (int64_t i = 0; i < n; ++i) {
        int tmp[ORC_NANG];
        orc_unpack_record(rec + i * ORC_REC, tmp, rad + i * ORC_NBLK);
        for (int a = 0; a < ORC_NANG; ++a) J[i * ORC_NANG + a] = tmp[a];
    }
}

/* ------------------------------------------------------------------ */
/* Encode (Algorithm 1 lines 2 and 4 with Section 4.1's settings).     */
/* x[n][128] already widened exactly to double.  For every vector:     */
/*   y = x * S  (row vector times matrix, S row-major S[i][j]);        */
/*   each block of 16 consecutive coordinates of y is one independent  */
/*   depth-4 polar transform;                                          */
/*   every angle is replaced by the index of its nearest centroid;     */
/*   r^(4) is rounded to binary16.                                     */
/* Angles of the whole vector are numbered level-major with the blocks */
/* side by side: level-1 angle j covers coordinates (2j, 2j+1), level  */
/* l angle j covers coordinates [j 2^l, (j+1) 2^l).                    */
/* Outputs (any may be NULL): rec[n][62], psi_out[n][120] (the exact   */
/* angles, for boundary-distance analysis), y_out[n][128].             */
/* ------------------------------------------------------------------ */
void orc_encode(const double *x, int64_t n, const double *S, const double *cb,
                uint8_t *rec, double *psi_out, double *y_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double y[ORC_D], psi[ORC_NANG], rblk[ORC_NBLK];
        int J[ORC_NANG];
        uint16_t rad[ORC_NBLK];
        const double *xi = x + i * ORC_D;
        for (int j = 0; j < ORC_D; ++j) {
            double acc = 0.0;
            for (int k = 0; k < ORC_D; ++k) acc += xi[k] * S[k * ORC_D + j];
            y[j] = acc;
        }
        /* blockwise depth-4 transform == depth-4 truncation of Polar on d=128 */
        orc_polar(y, ORC_D, ORC_L, psi, rblk);
        int off = 0, cnt = ORC_D / 2;
        for (int l = 1; l <= ORC_L; ++l) {
            for (int j = 0; j < cnt; ++j)
                J[off + j] = orc_quant(psi[off + j], cb + orc_cb_off[l], orc_cb_K[l]);
            off += cnt; cnt /= 2;
        }
        /* b_FPN = 16 (Section 4.1): binary16.  The paper is silent on radii beyond the format's range; reading:
           the stored radius saturates at the largest finite binary16 value, so that a block of extreme norm
           keeps its direction and stays finite instead of turning into infinity. */
        for (int b = 0; b < ORC_NBLK; ++b) rad[b] = orc_f64_to_f16(fmin(rblk[b], ORC_F16_MAX));
        if (rec) orc_pack_record(J, rad, rec + i * ORC_REC);
        if (psi_out) memcpy(psi_out + i * ORC_NANG, psi, sizeof(psi));
        if (y_out) memcpy(y_out + i * ORC_D, y, sizeof(y));
    }
}

/* DeQuant's loops for one record: r^(0) in the rotated domain (no S^T). */
static void orc_dequant_rotated_one(const uint8_t *rec, const double *cb, double *y)
{
    int J[ORC_NANG];
    uint16_t rad[ORC_NBLK];
    double psi[ORC_NANG], r[ORC_NBLK];
    orc_unpack_record(rec, J, rad);
    int off = 0, cnt = ORC_D / 2;
    for (int l = 1; l <= ORC_L; ++l) {
        for (int j = 0; j < cnt; ++j) psi[off + j] = cb[orc_cb_off[l] + J[off + j]];
        off += cnt; cnt /= 2;
    }
    for (int b = 0; b < ORC_NBLK; ++b) r[b] = orc_f16_to_f64(rad[b]);
    orc_polar_inverse(psi, r, ORC_D, ORC_L, y);
}

/* ------------------------------------------------------------------ */
/* Procedure DeQuant: records -> vectors.  rotated != 0 stops before   */
/* the trailing multiplication by S^T (output r^(0)); otherwise the    */
/* output is r^(0) * S^T, i.e. xhat_i = sum_j yhat_j S[i][j].          */
/* ------------------------------------------------------------------ */
void orc_decode(const uint8_t *rec, int64_t n, const double *S, const double *cb,
                int rotated, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double y[ORC_D];
        orc_dequant_rotated_one(rec + t * ORC_REC, cb, y);
        double *o = out + t * ORC_D;
        if (rotated) { memcpy(o, y, sizeof(y)); continue; }
        for (int i = 0; i < ORC_D; ++i) {
            double acc = 0.0;
            for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
            o[i] = acc;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Attention of one new query per sequence on the dequantised cache    */
/* (Eq. 5):  out = softmax(Khat q * scale)^T Vhat, every step double.  */
/*   q[B][Hq][128]; records k_rec, v_rec are [Hkv][plane_tokens][62];  */
/*   sequence b owns tokens [seq_start[b], seq_start[b]+ctx_len[b]) of */
/*   every head plane; query head h reads kv head h / (Hq/Hkv).        */
/* rotated == 0: the definition -- Khat, Vhat fully dequantised        */
/*   (including S^T), textbook two-pass softmax.                       */
/* rotated != 0: same quantity computed in the rotated domain:         */
/*   q' = q S, scores and weighted sum on r^(0) rows, result times     */
/*   S^T.  Equal to the former up to rounding because S is orthogonal. */
/* ctx_len[b] == 0 gives a zero output row.                            */
/* ------------------------------------------------------------------ */
void orc_attention(const double *q, int B, int Hq, int Hkv,
                   const uint8_t *k_rec, const uint8_t *v_rec,
                   const int64_t *seq_start, const int32_t *ctx_len,
                   int64_t plane_tokens, const double *S, const double *cb,
                   double scale, int rotated, double *out)
{
    int G = Hq / Hkv;
    int64_t pairs = (int64_t)B * Hkv;
    for (int64_t p = 0; p < pairs; ++p) {
        int b = (int)(p / Hkv), hk = (int)(p % Hkv);
        int64_t T = ctx_len[b];
        for (int g = 0; g < G; ++g)
            memset(out + ((int64_t)b * Hq + hk * G + g) * ORC_D, 0, sizeof(double) * ORC_D);
        if (T <= 0) continue;
        const uint8_t *kr = k_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC;
        const uint8_t *vr = v_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC;
        double *Kh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *Vh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *sc = (double *)malloc(sizeof(double) * T);
        /* DeQuant of every cached row (rows are independent) */
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            double y[ORC_D];
            orc_dequant_rotated_one(kr + t * ORC_REC, cb, y);
            if (rotated) memcpy(Kh + t * ORC_D, y, sizeof(y));
            else for (int i = 0; i < ORC_D; ++i) {
                double acc = 0.0;
                for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
                Kh[t * ORC_D + i] = acc;
            }
            orc_dequant_rotated_one(vr + t * ORC_REC, cb, y);
            if (rotated) memcpy(Vh + t * ORC_D, y, sizeof(y));
            else for (int i = 0; i < ORC_D; ++i) {
                double acc = 0.0;
                for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
                Vh[t * ORC_D + i] = acc;
            }
        }
        for (int g = 0; g < G; ++g) {
            const double *qh = q + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double *oh = out + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double qr[ORC_D], acc_o[ORC_D];
            if (rotated) {
                for (int j = 0; j < ORC_D; ++j) {
                    double a = 0.0;
                    for (int k = 0; k < ORC_D; ++k) a += qh[k] * S[k * ORC_D + j];
                    qr[j] = a;
                }
            } else memcpy(qr, qh, sizeof(qr));
            double mx = -INFINITY;
            for (int64_t t = 0; t < T; ++t) {
                double s = 0.0;
                for (int j = 0; j < ORC_D; ++j) s += Kh[t * ORC_D + j] * qr[j];
                sc[t] = s * scale;
                if (sc[t] > mx) mx = sc[t];
            }
            double den = 0.0;
            for (int64_t t = 0; t < T; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
            for (int j = 0; j < ORC_D; ++j) acc_o[j] = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double w = sc[t] / den;
                for (int j = 0; j < ORC_D; ++j) acc_o[j] += w * Vh[t * ORC_D + j];
            }
            if (rotated) {
                for (int i = 0; i < ORC_D; ++i) {
                    double a = 0.0;
                    for (int j = 0; j < ORC_D; ++j) a += acc_o[j] * S[i * ORC_D + j];
                    oh[i] = a;
                }
            } else memcpy(oh, acc_o, sizeof(acc_o));
        }
        free(Kh); free(Vh); free(sc);
    }
}

/* ------------------------------------------------------------------ */
/* Attention over a quantised prefix plus an unquantised recent window  */
/* (Section 5.3: the keys and values streamed in during generation are  */
/* kept in 16 bits, only the prompt's are quantised).  One softmax over */
/* the concatenation: the first ctx_len[b] rows are the DeQuant of the  */
/* cached records (Eq. 5), the next win_len[b] rows are the window's    */
/* vectors as given.  win_k, win_v: [B][Hkv][win_cap][128].             */
/* No rows at all gives a zero output row.                              */
/* ------------------------------------------------------------------ */
void orc_attention_hybrid(const double *q, int B, int Hq, int Hkv,
                          const uint8_t *k_rec, const uint8_t *v_rec,
                          const int64_t *seq_start, const int32_t *ctx_len,
                          int64_t plane_tokens, const double *win_k, const double *win_v,
                          const int32_t *win_len, int64_t win_cap,
                          const double *S, const double *cb, double scale, double *out)
{
    int G = Hq / Hkv;
    for (int b = 0; b < B; ++b)
        for (int hk = 0; hk < Hkv; ++hk) {
            int64_t T = ctx_len[b] > 0 ? ctx_len[b] : 0, W = win_len[b] > 0 ? win_len[b] : 0, N = T + W;
            for (int g = 0; g < G; ++g)
                memset(out + ((int64_t)b * Hq + hk * G + g) * ORC_D, 0, sizeof(double) * ORC_D);
            if (N == 0) continue;
            double *Kh = (double *)malloc(sizeof(double) * N * ORC_D);
            double *Vh = (double *)malloc(sizeof(double) * N * ORC_D);
            double *sc = (double *)malloc(sizeof(double) * N);
            const uint8_t *kr = k_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC;
            const uint8_t *vr = v_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC;
#pragma omp parallel for schedule(static)
            for (int64_t t = 0; t < T; ++t) { /* procedure DeQuant, trailing S^T included */
                double y[ORC_D];
                orc_dequant_rotated_one(kr + t * ORC_REC, cb, y);
                for (int i = 0; i < ORC_D; ++i) {
                    double acc = 0.0;
                    for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
                    Kh[t * ORC_D + i] = acc;
                }
                orc_dequant_rotated_one(vr + t * ORC_REC, cb, y);
                for (int i = 0; i < ORC_D; ++i) {
                    double acc = 0.0;
                    for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
                    Vh[t * ORC_D + i] = acc;
                }
            }
            const double *wk = win_k + ((int64_t)b * Hkv + hk) * win_cap * ORC_D;
            const double *wv = win_v + ((int64_t)b * Hkv + hk) * win_cap * ORC_D;
            for (int64_t t = 0; t < W; ++t) {
                memcpy(Kh + (T + t) * ORC_D, wk + t * ORC_D, sizeof(double) * ORC_D);
                memcpy(Vh + (T + t) * ORC_D, wv + t * ORC_D, sizeof(double) * ORC_D);
            }
            for (int g = 0; g < G; ++g) {
                const double *qh = q + ((int64_t)b * Hq + hk * G + g) * ORC_D;
                double *oh = out + ((int64_t)b * Hq + hk * G + g) * ORC_D;
                double mx = -INFINITY, den = 0.0;
                for (int64_t t = 0; t < N; ++t) {
                    double s = 0.0;
                    for (int j = 0; j < ORC_D; ++j) s += Kh[t * ORC_D + j] * qh[j];
                    sc[t] = s * scale;
                    if (sc[t] > mx) mx = sc[t];
                }
                for (int64_t t = 0; t < N; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
                for (int64_t t = 0; t < N; ++t) {
                    double w = sc[t] / den;
                    for (int j = 0; j < ORC_D; ++j) oh[j] += w * Vh[t * ORC_D + j];
                }
            }
            free(Kh); free(Vh); free(sc);
        }
}

/* Exact attention on unquantised K, V (Eq. 4), for reporting the       */
/* approximation error only.  parity unpinned against the paper (it     */
/* prints no bound relating Eq. 5 to Eq. 4); it is plain softmax.       */
void orc_attention_exact(const double *q, const double *K, const double *V,
                         int64_t T, int G, double scale, double *out)
{
    double *sc = (double *)malloc(sizeof(double) * T);
    for (int g = 0; g < G; ++g) {
        const double *qh = q + (int64_t)g * ORC_D;
        double mx = -INFINITY, den = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double s = 0.0;
            for (int j = 0; j < ORC_D; ++j) s += K[t * ORC_D + j] * qh[j];
            sc[t] = s * scale;
            if (sc[t] > mx) mx = sc[t];
        }
        for (int64_t t = 0; t < T; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
        for (int j = 0; j < ORC_D; ++j) out[g * ORC_D + j] = 0.0;
        for (int64_t t = 0; t < T; ++t)
            for (int j = 0; j < ORC_D; ++j) out[g * ORC_D + j] += sc[t] / den * V[t * ORC_D + j];
    }
    free(sc);
}

/* ------------------------------------------------------------------ */
/* Full-depth recursion (Definition 1 and procedure Polar of Algorithm */
/* 1 run to level log2 d = 7; Section 4's memory count: one radius per */
/* vector plus the angle codes).  Levels 1..4 keep Section 4.1's bit   */
/* widths and codebooks; levels 5, 6, 7 -- the 4 + 2 + 1 angles that   */
/* join the 8 block radii -- take bits[0..2] bits each (the codebook   */
/* size of a level is free: remark after Theorem 1) and the codebooks  */
/* cbt[3][8]: row l-5 holds the 2^bits[l-5] centroids of level l.      */
/*                                                                     */
/* Canonical deep record (50 bytes): bytes 0..45 as in the 62-byte     */
/* record (levels 1..4); bytes 46..47 a 16-bit little-endian word with */
/* the level-5 codes j = 0..3 at bits [j b5, (j+1) b5), the level-6    */
/* codes j = 0, 1 at bits [4 b5 + j b6, ...), the level-7 code at bit  */
/* 4 b5 + 2 b6 (unused high bits zero; 4 b5 + 2 b6 + b7 <= 16);        */
/* bytes 48..49 the binary16 radius r^(7) = |y|, little endian.        */
/* Pinned by: levels 1..4 identical to the depth-4 record, DeQuant of  */
/* the record lies on the sphere of the stored radius, DeQuant equals  */
/* the inverse transform fed with the centroids of the unpacked codes, */
/* angle statistics of levels 5..7 against Lemma 2, predicted error.   */
/* ------------------------------------------------------------------ */
#define ORC_REC_DEEP 50
#define ORC_NANG_DEEP 127    /* 64 + 32 + 16 + 8 + 4 + 2 + 1 */
#define ORC_L_DEEP 7

int orc_upper_codebooks(const int *bits, double *cbt)
{
    double bnd[9];
    for (int l = 5; l <= 7; ++l) {
        int b = bits[l - 5];
        if (b < 1 || b > 3) return -1;
        for (int k = 0; k < 8; ++k) cbt[(l - 5) * 8 + k] = 0.0;
        if (orc_codebook(l, 1 << b, cbt + (l - 5) * 8, bnd)) return -1;
    }
    return (4 * bits[0] + 2 * bits[1] + bits[2] <= 16) ? 0 : -1;
}

/* J: the 127 codes level-major; rad: binary16 bits of r^(7) */
static void orc_pack_record_deep(const int *J, uint16_t rad, const int *bits, uint8_t *rec)
{
    uint8_t base[ORC_REC];
    uint16_t none[ORC_NBLK] = {0};
    orc_pack_record(J, none, base);
    memcpy(rec, base, 46);
    unsigned word = 0;
    int pos = 0, at = ORC_NANG;
    for (int l = 5; l <= 7; ++l)
        for (int j = 0; j < (ORC_D >> l); ++j) {
            word |= (unsigned)J[at++] << pos;
            pos += bits[l - 5];
        }
    rec[46] = (uint8_t)(word & 0xFF); rec[47] = (uint8_t)(word >> 8);
    rec[48] = (uint8_t)(rad & 0xFF);  rec[49] = (uint8_t)(rad >> 8);
}

static void orc_unpack_record_deep(const uint8_t *rec, const int *bits, int *J, uint16_t *rad)
{
    uint8_t base[ORC_REC];
    uint16_t none[ORC_NBLK];
    memset(base, 0, sizeof(base));
    memcpy(base, rec, 46);
    orc_unpack_record(base, J, none);
    unsigned word = (unsigned)rec[46] | ((unsigned)rec[47] << 8);
    int pos = 0, at = ORC_NANG;
    for (int l = 5; l <= 7; ++l)
        for (int j = 0; j < (ORC_D >> l); ++j) {
            J[at++] = (int)((word >> pos) & ((1u << bits[l - 5]) - 1u));
            pos += bits[l - 5];
        }
    *rad = (uint16_t)(rec[48] | (rec[49] << 8));
}

void orc_unpack_deep(const uint8_t *rec, int64_t n, const int *bits, int32_t *J, uint16_t *rad)
{
    for (int64_t i = 0; i < n; ++i) {
        int tmp[ORC_NANG_DEEP];
        orc_unpack_record_deep(rec + i * ORC_REC_DEEP, bits, tmp, rad + i);
        for (int a = 0; a < ORC_NANG_DEEP; ++a) J[i * ORC_NANG_DEEP + a] = tmp[a];
    }
}

/* centroid list and size of level l = 1..7 */
static const double *orc_level_centroids(int l, const double *cb, const int *bits, const double *cbt, int *K)
{
    if (l <= ORC_L) { *K = orc_cb_K[l]; return cb + orc_cb_off[l]; }
    *K = 1 << bits[l - 5];
    return cbt + (l - 5) * 8;
}

/* Encode at full depth: y = x S, procedure Polar with L = 7, procedure Quant per level, */
/* the one radius r^(7) rounded to binary16.  Outputs (any may be NULL): rec[n][50],     */
/* psi_out[n][127] (exact angles, level-major), y_out[n][128].                           */
void orc_encode_deep(const double *x, int64_t n, const double *S, const double *cb,
                     const int *bits, const double *cbt,
                     uint8_t *rec, double *psi_out, double *y_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double y[ORC_D], psi[ORC_NANG_DEEP], r7[1];
        int J[ORC_NANG_DEEP];
        const double *xi = x + i * ORC_D;
        for (int j = 0; j < ORC_D; ++j) {
            double acc = 0.0;
            for (int k = 0; k < ORC_D; ++k) acc += xi[k] * S[k * ORC_D + j];
            y[j] = acc;
        }
        orc_polar(y, ORC_D, ORC_L_DEEP, psi, r7);
        int off = 0, cnt = ORC_D / 2;
        for (int l = 1; l <= ORC_L_DEEP; ++l) {
            int K;
            const double *theta = orc_level_centroids(l, cb, bits, cbt, &K);
            for (int j = 0; j < cnt; ++j) J[off + j] = orc_quant(psi[off + j], theta, K);
            off += cnt; cnt /= 2;
        }
        if (rec) orc_pack_record_deep(J, orc_f64_to_f16(fmin(r7[0], ORC_F16_MAX)), bits, rec + i * ORC_REC_DEEP); /* saturates like the block radii */
        if (psi_out) memcpy(psi_out + i * ORC_NANG_DEEP, psi, sizeof(psi));
        if (y_out) memcpy(y_out + i * ORC_D, y, sizeof(y));
    }
}

/* DeQuant's loops for one deep record: r^(0) in the rotated domain. */
static void orc_dequant_rotated_one_deep(const uint8_t *rec, const double *cb, const int *bits,
                                         const double *cbt, double *y)
{
    int J[ORC_NANG_DEEP];
    uint16_t rad;
    double psi[ORC_NANG_DEEP], r[1];
    orc_unpack_record_deep(rec, bits, J, &rad);
    int off = 0, cnt = ORC_D / 2;
    for (int l = 1; l <= ORC_L_DEEP; ++l) {
        int K;
        const double *theta = orc_level_centroids(l, cb, bits, cbt, &K);
        for (int j = 0; j < cnt; ++j) psi[off + j] = theta[J[off + j]];
        off += cnt; cnt /= 2;
    }
    r[0] = orc_f16_to_f64(rad);
    orc_polar_inverse(psi, r, ORC_D, ORC_L_DEEP, y);
}

void orc_decode_deep(const uint8_t *rec, int64_t n, const double *S, const double *cb,
                     const int *bits, const double *cbt, int rotated, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double y[ORC_D];
        orc_dequant_rotated_one_deep(rec + t * ORC_REC_DEEP, cb, bits, cbt, y);
        double *o = out + t * ORC_D;
        if (rotated) { memcpy(o, y, sizeof(y)); continue; }
        for (int i = 0; i < ORC_D; ++i) {
            double acc = 0.0;
            for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
            o[i] = acc;
        }
    }
}

/* Eq. 5 on deep records: every cached row is dequantised (including S^T), then the      */
/* textbook two-pass softmax; layout of the arguments as in orc_attention with 50-byte   */
/* records.                                                                              */
void orc_attention_deep(const double *q, int B, int Hq, int Hkv,
                        const uint8_t *k_rec, const uint8_t *v_rec,
                        const int64_t *seq_start, const int32_t *ctx_len,
                        int64_t plane_tokens, const double *S, const double *cb,
                        const int *bits, const double *cbt, double scale, double *out)
{
    int G = Hq / Hkv;
    for (int64_t p = 0; p < (int64_t)B * Hkv; ++p) {
        int b = (int)(p / Hkv), hk = (int)(p % Hkv);
        int64_t T = ctx_len[b];
        for (int g = 0; g < G; ++g)
            memset(out + ((int64_t)b * Hq + hk * G + g) * ORC_D, 0, sizeof(double) * ORC_D);
        if (T <= 0) continue;
        const uint8_t *kr = k_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC_DEEP;
        const uint8_t *vr = v_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * ORC_REC_DEEP;
        double *Kh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *Vh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *sc = (double *)malloc(sizeof(double) * T);
        orc_decode_deep(kr, T, S, cb, bits, cbt, 0, Kh);
        orc_decode_deep(vr, T, S, cb, bits, cbt, 0, Vh);
        for (int g = 0; g < G; ++g) {
            const double *qh = q + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double *oh = out + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double mx = -INFINITY;
            for (int64_t t = 0; t < T; ++t) {
                double s = 0.0;
                for (int j = 0; j < ORC_D; ++j) s += Kh[t * ORC_D + j] * qh[j];
                sc[t] = s * scale;
                if (sc[t] > mx) mx = sc[t];
            }
            double den = 0.0;
            for (int64_t t = 0; t < T; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
            for (int64_t t = 0; t < T; ++t) {
                double w = sc[t] / den;
                for (int j = 0; j < ORC_D; ++j) oh[j] += w * Vh[t * ORC_D + j];
            }
        }
        free(Kh); free(Vh); free(sc);
    }
}

/* ------------------------------------------------------------------ */
/* Online codebook (Section 4.1: 1-D k-means on the angles of the       */
/* polar-transformed inputs; Eq. 3 with the samples in place of the     */
/* density).  All angles of all n vectors of a level form one sample    */
/* set; `iterations` rounds of the k-means (Lloyd) update from the      */
/* centroids in cb_init: every angle goes to its nearest centroid       */
/* (linear distance, lowest index on ties, as procedure Quant), every   */
/* centroid moves to the mean of its angles; a centroid without angles  */
/* stays.  Reading: the paper seeds with k-means++ (randomised); here   */
/* the seed is cb_init (the analytic codebook, say), which makes the    */
/* result a function of the data alone.                                 */
/* ------------------------------------------------------------------ */
void orc_fit_codebooks(const double *x, int64_t n, const double *S, const double *cb_init,
                       int iterations, double *cb_out)
{
    double *psi = (double *)malloc(sizeof(double) * (size_t)n * ORC_NANG);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double y[ORC_D], rblk[ORC_NBLK];
        const double *xi = x + i * ORC_D;
        for (int j = 0; j < ORC_D; ++j) {
            double acc = 0.0;
            for (int k = 0; k < ORC_D; ++k) acc += xi[k] * S[k * ORC_D + j];
            y[j] = acc;
        }
        orc_polar(y, ORC_D, ORC_L, psi + i * ORC_NANG, rblk);
    }
    memcpy(cb_out, cb_init, sizeof(double) * 28);
    int off = 0, cnt = ORC_D / 2;
    for (int l = 1; l <= ORC_L; ++l) {
        int K = orc_cb_K[l];
        double *c = cb_out + orc_cb_off[l];
        for (int it = 0; it < iterations; ++it) {
            double sum[16];
            int64_t num[16];
            for (int k = 0; k < K; ++k) { sum[k] = 0.0; num[k] = 0; }
            for (int64_t i = 0; i < n; ++i)
                for (int j = 0; j < cnt; ++j) {
                    double a = psi[i * ORC_NANG + off + j];
                    int k = orc_quant(a, c, K);
                    sum[k] += a;
                    num[k] += 1;
                }
            for (int k = 0; k < K; ++k)
                if (num[k] > 0) c[k] = sum[k] / (double)num[k];
        }
        off += cnt; cnt /= 2;
    }
    free(psi);
}

/* ================================================================== */
/* General format: any recursion depth L in 1..7 and any number of     */
/* bits per level (Definition 1 recurses to log2 d; the remark after    */
/* Theorem 1 leaves the codebook size of each level free; Section 4.1   */
/* is the instance L = 4, bits 4/2/2/2).  d = 128.                      */
/*   bits[l-1]   bits of level l, 1..4 (level 1 up to 6)               */
/*   cbg         centroids of levels 1..L one after another, level l   */
/*               holding 2^bits[l-1] entries                           */
/*   record      the codes of level 1 (64 of them, in coordinate       */
/*               order), then level 2 (32), ..., each bits[l-1] wide,  */
/*               written into one little-endian bit stream (bit p of   */
/*               the stream is bit p & 7 of byte p >> 3), padded to a  */
/*               whole byte; then the 128 >> L radii r^(L) as          */
/*               little-endian binary16 (saturating like the others).  */
/* Pinned by: L = 4 with bits 4/2/2/2 gives the codes, radii and       */
/* decoded vectors of the Section 4.1 functions above; exact inverse   */
/* with exact angles at every depth (orc_polar pins); Lloyd-Max        */
/* conditions of the larger codebooks by independent quadrature; the   */
/* predicted reconstruction error; textbook softmax.                   */
/* ================================================================== */
static int orc_general_nang(int L)
{
    int n = 0;
    for (int l = 1; l <= L; ++l) n += ORC_D >> l;
    return n;
}

int orc_general_record_bytes(int L, const int *bits)
{
    if (L < 1 || L > 7) return -1;
    int nbits = 0;
    for (int l = 1; l <= L; ++l) {
        if (bits[l - 1] < 1 || bits[l - 1] > 6) return -1;
        nbits += (ORC_D >> l) * bits[l - 1];
    }
    return (nbits + 7) / 8 + 2 * (ORC_D >> L);
}

/* Lloyd-Max codebooks of Lemma 2's densities for the given sizes (level 1: equal cells). */
int orc_general_codebooks(int L, const int *bits, double *cbg)
{
    double bnd[65];
    int off = 0;
    for (int l = 1; l <= L; ++l) {
        int K = 1 << bits[l - 1];
        if (orc_codebook(l, K, cbg + off, bnd)) return -1;
        off += K;
    }
    return 0;
}

static void orc_put_bits(uint8_t *stream, int pos, int width, int v)
{
    for (int i = 0; i < width; ++i)
        if ((v >> i) & 1) stream[(pos + i) >> 3] |= (uint8_t)(1u << ((pos + i) & 7));
}

static int orc_get_bits(const uint8_t *stream, int pos, int width)
{
    int v = 0;
    for (int i = 0; i < width; ++i) v |= ((stream[(pos + i) >> 3] >> ((pos + i) & 7)) & 1) << i;
    return v;
}

/* x[n][128] -> rec[n][record bytes]; psi_out[n][nang] (exact angles, level-major) and J_out[n][nang] optional */
void orc_encode_general(const double *x, int64_t n, const double *S, int L, const int *bits, const double *cbg,
                        uint8_t *rec, double *psi_out, int32_t *J_out)
{
    const int nang = orc_general_nang(L), nrad = ORC_D >> L, rb = orc_general_record_bytes(L, bits);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double y[ORC_D], psi[ORC_NANG_DEEP], r[ORC_D];
        const double *xi = x + i * ORC_D;
        for (int j = 0; j < ORC_D; ++j) {
            double acc = 0.0;
            for (int k = 0; k < ORC_D; ++k) acc += xi[k] * S[k * ORC_D + j];
            y[j] = acc;
        }
        orc_polar(y, ORC_D, L, psi, r);
        uint8_t *ri = rec + i * rb;
        memset(ri, 0, (size_t)rb);
        int off = 0, cnt = ORC_D / 2, cboff = 0, pos = 0;
        for (int l = 1; l <= L; ++l) {
            int K = 1 << bits[l - 1];
            for (int j = 0; j < cnt; ++j) {
                int code = orc_quant(psi[off + j], cbg + cboff, K);
                orc_put_bits(ri, pos, bits[l - 1], code);
                pos += bits[l - 1];
                if (J_out) J_out[i * nang + off + j] = code;
            }
            off += cnt; cnt /= 2; cboff += K;
        }
        uint8_t *rr = ri + (pos + 7) / 8;
        for (int b = 0; b < nrad; ++b) {
            uint16_t h = orc_f64_to_f16(fmin(r[b], ORC_F16_MAX));
            rr[2 * b] = (uint8_t)(h & 0xFF);
            rr[2 * b + 1] = (uint8_t)(h >> 8);
        }
        if (psi_out) memcpy(psi_out + i * nang, psi, sizeof(double) * nang);
    }
}

/* DeQuant's loops for one general record: r^(0) in the rotated domain */
static void orc_dequant_rotated_general(const uint8_t *rec, int L, const int *bits, const double *cbg, double *y)
{
    double psi[ORC_NANG_DEEP], r[ORC_D];
    const int nrad = ORC_D >> L;
    int off = 0, cnt = ORC_D / 2, cboff = 0, pos = 0;
    for (int l = 1; l <= L; ++l) {
        for (int j = 0; j < cnt; ++j) {
            psi[off + j] = cbg[cboff + orc_get_bits(rec, pos, bits[l - 1])];
            pos += bits[l - 1];
        }
        off += cnt; cnt /= 2; cboff += 1 << bits[l - 1];
    }
    const uint8_t *rr = rec + (pos + 7) / 8;
    for (int b = 0; b < nrad; ++b) r[b] = orc_f16_to_f64((uint16_t)(rr[2 * b] | (rr[2 * b + 1] << 8)));
    orc_polar_inverse(psi, r, ORC_D, L, y);
}

/* records -> vectors; rotated != 0 stops before the trailing S^T */
void orc_decode_general(const uint8_t *rec, int64_t n, const double *S, int L, const int *bits, const double *cbg,
                        int rotated, double *out)
{
    const int rb = orc_general_record_bytes(L, bits);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double y[ORC_D];
        orc_dequant_rotated_general(rec + t * rb, L, bits, cbg, y);
        double *o = out + t * ORC_D;
        if (rotated) { memcpy(o, y, sizeof(y)); continue; }
        for (int i = 0; i < ORC_D; ++i) {
            double acc = 0.0;
            for (int j = 0; j < ORC_D; ++j) acc += y[j] * S[i * ORC_D + j];
            o[i] = acc;
        }
    }
}

/* Eq. 5 on general records: the definition (rows fully dequantised, textbook two-pass softmax).
   Shapes as orc_attention; records are [Hkv][plane_tokens][record bytes]. */
void orc_attention_general(const double *q, int B, int Hq, int Hkv, const uint8_t *k_rec, const uint8_t *v_rec,
                           const int64_t *seq_start, const int32_t *ctx_len, int64_t plane_tokens, const double *S,
                           int L, const int *bits, const double *cbg, double scale, double *out)
{
    const int G = Hq / Hkv, rb = orc_general_record_bytes(L, bits);
    for (int64_t p = 0; p < (int64_t)B * Hkv; ++p) {
        int b = (int)(p / Hkv), hk = (int)(p % Hkv);
        int64_t T = ctx_len[b];
        for (int g = 0; g < G; ++g)
            memset(out + ((int64_t)b * Hq + hk * G + g) * ORC_D, 0, sizeof(double) * ORC_D);
        if (T <= 0) continue;
        double *Kh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *Vh = (double *)malloc(sizeof(double) * T * ORC_D);
        double *w = (double *)malloc(sizeof(double) * T);
        orc_decode_general(k_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * rb, T, S, L, bits, cbg, 0, Kh);
        orc_decode_general(v_rec + ((int64_t)hk * plane_tokens + seq_start[b]) * rb, T, S, L, bits, cbg, 0, Vh);
        for (int g = 0; g < G; ++g) {
            const double *qh = q + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double *o = out + ((int64_t)b * Hq + hk * G + g) * ORC_D;
            double mx = -INFINITY, sum = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int i = 0; i < ORC_D; ++i) acc += qh[i] * Kh[t * ORC_D + i];
                w[t] = acc * scale;
                if (w[t] > mx) mx = w[t];
            }
            for (int64_t t = 0; t < T; ++t) { w[t] = exp(w[t] - mx); sum += w[t]; }
            for (int64_t t = 0; t < T; ++t)
                for (int i = 0; i < ORC_D; ++i) o[i] += (w[t] / sum) * Vh[t * ORC_D + i];
        }
        free(Kh); free(Vh); free(w);
    }
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
