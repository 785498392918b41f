/*
 * pq_host.hip -- host side of libpolarquant: context creation (random
 * rotation S, Lloyd-Max codebooks of the closed-form angle densities, lookup
 * tables), per-device upload of the constants, small utilities.
 *
 * Everything here is double precision on the CPU and runs once per model
 * (Section 4.1: S and the offline codebook are shared by all layers, heads
 * and prompts).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <new>
#include <vector>

#include "pq_common.h"

namespace {

const double kPi = 3.14159265358979323846264338327950288;

/* ---- counter-based Gaussian generator: splitmix64 finaliser + Box-Muller ---- */
uint64_t splitmix_finalise(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

double uniform_open01(uint64_t seed_mixed, uint64_t counter)
{
    uint64_t bits = splitmix_finalise(seed_mixed + (counter + 1) * 0x9E3779B97F4A7C15ULL);
    return ((double)(bits >> 11) + 0.5) * 0x1.0p-53;
}

void fill_gaussian(uint64_t seed, int d, std::vector<double> &G)
{
    const uint64_t sm = splitmix_finalise(seed);
    G.resize((size_t)d * d);
    for (size_t c = 0; c < (size_t)d * d; ++c) {
        double u1 = uniform_open01(sm, 2 * c), u2 = uniform_open01(sm, 2 * c + 1);
        G[c] = sqrt(-2.0 * log(u1)) * cos(2.0 * kPi * u2);
    }
}

/* ---- S = Q of the QR factorisation with positive diag(R): the columns of G
 * orthonormalised in order (modified Gram-Schmidt, each projection pass done
 * twice so that orthogonality holds to rounding). ---- */
bool orthonormalise_columns(const std::vector<double> &G, int d, double *S)
{
    std::vector<double> col(d);
    for (int j = 0; j < d; ++j) {
        for (int i = 0; i < d; ++i) col[i] = G[(size_t)i * d + j];
        for (int pass = 0; pass < 2; ++pass)
            for (int p = 0; p < j; ++p) {
                double dot = 0.0;
                for (int i = 0; i < d; ++i) dot += S[(size_t)i * d + p] * col[i];
                for (int i = 0; i < d; ++i) col[i] -= dot * S[(size_t)i * d + p];
            }
        double nrm = 0.0;
        for (int i = 0; i < d; ++i) nrm += col[i] * col[i];
        nrm = sqrt(nrm);
        if (!(nrm > 1e-300)) return false;
        for (int i = 0; i < d; ++i) S[(size_t)i * d + j] = col[i] / nrm;
    }
    return true;
}

double orthogonality_defect(const double *S, int d)
{
    double worst = 0.0;
    for (int a = 0; a < d; ++a)
        for (int b = a; b < d; ++b) {
            double dot = 0.0;
            for (int i = 0; i < d; ++i) dot += S[(size_t)i * d + a] * S[(size_t)i * d + b];
            double e = fabs(dot - (a == b ? 1.0 : 0.0));
            if (e > worst) worst = e;
        }
    return worst;
}

/* ---- Lloyd-Max quantiser of f_l(psi) ~ sin^m(2 psi), m = 2^(l-1) - 1 (Lemma 2),
 * on [0, pi/2], with closed-form moments: for odd m
 *   sin^m(u) = 2^(1-m) * sum_{k=0}^{(m-1)/2} (-1)^((m-1)/2-k) C(m,k) sin((m-2k) u),
 * so the integrals of sin^m(2 psi) and psi*sin^m(2 psi) are finite sums of
 * elementary antiderivatives. ---- */
struct SinPower {
    int terms;
    double coef[32], freq[32]; /* sin^m(2 psi) = sum coef[k] * sin(freq[k] * psi); m <= 63 */
};

SinPower make_sin_power(int m)
{
    SinPower sp;
    sp.terms = (m + 1) / 2;
    double binom = 1.0; /* C(m, k) */
    for (int k = 0; k < sp.terms; ++k) {
        double sign = (((m - 1) / 2 - k) & 1) ? -1.0 : 1.0;
        sp.coef[k] = sign * binom * ldexp(1.0, 1 - m);
        sp.freq[k] = 2.0 * (m - 2 * k);
        binom = binom * (m - k) / (k + 1);
    }
    return sp;
}

double mass_antiderivative(const SinPower &sp, double x) /* int sin^m(2x) dx */
{
    double acc = 0.0;
    for (int k = 0; k < sp.terms; ++k) acc += sp.coef[k] * (-cos(sp.freq[k] * x) / sp.freq[k]);
    return acc;
}

double first_moment_antiderivative(const SinPower &sp, double x) /* int x sin^m(2x) dx */
{
    double acc = 0.0;
    for (int k = 0; k < sp.terms; ++k) {
        double a = sp.freq[k];
        acc += sp.coef[k] * (-x * cos(a * x) / a + sin(a * x) / (a * a));
    }
    return acc;
}

void lloyd_max_level(int level, double *centroids /*K*/, double *boundaries /*K+1*/, int K = 4)
{
    const int m_pow = (1 << (level - 1)) - 1;
    const SinPower sp = make_sin_power(m_pow);
    const double lo = 0.0, hi = kPi / 2.0;
    const double total = mass_antiderivative(sp, hi) - mass_antiderivative(sp, lo);
    for (int k = 0; k < K; ++k) centroids[k] = hi * (k + 0.5) / K;
    for (int it = 0; it < 200000; ++it) {
        boundaries[0] = lo; boundaries[K] = hi;
        for (int k = 1; k < K; ++k) boundaries[k] = 0.5 * (centroids[k - 1] + centroids[k]);
        double moved = 0.0;
        for (int k = 0; k < K; ++k) {
            double mass = mass_antiderivative(sp, boundaries[k + 1]) - mass_antiderivative(sp, boundaries[k]);
            double mom = first_moment_antiderivative(sp, boundaries[k + 1]) - first_moment_antiderivative(sp, boundaries[k]);
            if (!(mass > 1e-7 * total)) {
                /* a cell far out in the tail of a high power (the outer cells of eight at level 7 hold 1e-20 of the
                   mass): the alternating sum cancels there, so the cell is integrated numerically instead
                   (composite Simpson on sin^m(2 psi) itself, all terms positive) */
                const int N = 2048;
                const double a = boundaries[k], h = (boundaries[k + 1] - a) / N;
                mass = 0.0; mom = 0.0;
                for (int i = 0; i <= N; ++i) {
                    const double x = a + h * i, w = (i == 0 || i == N) ? 1.0 : ((i & 1) ? 4.0 : 2.0);
                    const double g = pow(sin(2.0 * x), (double)m_pow);
                    mass += w * g;
                    mom += w * g * x;
                }
                mass *= h / 3.0; mom *= h / 3.0;
            }
            double c = mass > 0.0 ? mom / mass : 0.5 * (boundaries[k] + boundaries[k + 1]);
            moved = fmax(moved, fabs(c - centroids[k]));
            centroids[k] = c;
        }
        if (moved < 1e-15) break;
    }
    boundaries[0] = lo; boundaries[K] = hi;
    for (int k = 1; k < K; ++k) boundaries[k] = 0.5 * (centroids[k - 1] + centroids[k]);
}

} // namespace

/* the same quantiser for the other files of the library (the general format builds codebooks of other sizes) */
void pq_lloyd_max(int level, int K, double *centroids, double *boundaries) { lloyd_max_level(level, centroids, boundaries, K); }

namespace {

/* ---- binary16 / bfloat16 from double, round to nearest even ---- */
uint16_t to_binary16(double v)
{
    /* bit-level conversion of a finite double with one rounding step */
    uint64_t u;
    memcpy(&u, &v, 8);
    uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    int exp = (int)((u >> 52) & 0x7FF) - 1023;
    uint64_t frac = (u & 0xFFFFFFFFFFFFFULL) | (1ULL << 52); /* 1.frac, 53 bits */
    if (((u >> 52) & 0x7FF) == 0) return sign;             /* zero / double subnormal */
    if (exp > 15) return (uint16_t)(sign | 0x7C00u);
    int drop = 42;                                          /* keep 11 significant bits */
    if (exp < -14) drop += -14 - exp;                       /* binary16 subnormal: fewer bits */
    if (drop > 63) return sign;
    uint64_t kept = frac >> drop, rest = frac & ((1ULL << drop) - 1), half = 1ULL << (drop - 1);
    if (rest > half || (rest == half && (kept & 1))) kept += 1;
    if (exp < -14) return (uint16_t)(sign | (uint16_t)kept); /* kept == 1024 becomes the smallest normal */
    if (kept == 2048) { kept = 1024; exp += 1; if (exp > 15) return (uint16_t)(sign | 0x7C00u); }
    return (uint16_t)(sign | (uint16_t)((exp + 15) << 10) | (uint16_t)(kept - 1024));
}

uint32_t pack_h2(double lo, double hi) { return (uint32_t)to_binary16(lo) | ((uint32_t)to_binary16(hi) << 16); }

uint16_t to_bfloat16(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    /* the double -> float step is exact for the values used here or loses
       bits far below bf16's 8-bit significand; round the float to bf16 */
    uint32_t rounded = u + 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(rounded >> 16);
}

double from_bfloat16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

double from_binary16(uint16_t h)
{
    int e = (h >> 10) & 31, m = h & 1023;
    double v = e == 0 ? ldexp((double)m, -24) : ldexp(1024.0 + m, e - 25);
    return (h & 0x8000) ? -v : v;
}

/* Monotone map of an angle in [0, 2 pi) to [0, 4): quadrant number plus the share of the
   second coordinate (even quadrants) or of the first (odd quadrants) in |x| + |y|. */
double pseudo_angle(double psi)
{
    const double x = cos(psi), y = sin(psi), a = fabs(x), b = fabs(y);
    const int sa = x < 0, sb = y < 0, f = sa ^ sb, Q = 2 * sb + f;
    return Q + (f ? a : b) / (a + b);
}

void build_tables(pq_ctx *ctx)
{
    PqDeviceConsts &c = ctx->host_consts;
    memset(&c, 0, sizeof(c));
    for (int l = 1; l <= 4; ++l) {
        const double *bnd = ctx->boundaries[l - 1];
        if (l == 1) {
            c.tan_b[0][0] = (float)tan(kPi / 8.0);
            c.tan_b[0][1] = 1.0f;
            c.tan_b[0][2] = (float)tan(3.0 * kPi / 8.0);
        } else {
            c.tan_b[l - 1][0] = (float)tan(bnd[1]);
            /* analytic codebooks: the middle boundary is pi/4 by symmetry of the density */
            c.tan_b[l - 1][1] = ctx->general_codebooks ? (float)tan(bnd[2]) : 1.0f;
            c.tan_b[l - 1][2] = (float)tan(bnd[3]);
        }
    }
    c.depth = ctx->depth;
    if (ctx->depth == 7)
        for (int l = 0; l < 3; ++l) {
            const int K = 1 << ctx->upper_bits[l];
            c.up_bits[l] = ctx->upper_bits[l];
            for (int k = 0; k < K - 1; ++k) {
                const double t = tan(ctx->upper_boundaries[l][k + 1]);
                c.up_tan2[l][k] = (float)(t * t);
            }
            for (int k = 0; k < K; ++k) {
                c.up_cs[l][k][0] = (float)cos(ctx->upper_centroids[l][k]);
                c.up_cs[l][k][1] = (float)sin(ctx->upper_centroids[l][k]);
            }
        }
    c.general = ctx->general_codebooks ? 1 : 0;
    if (ctx->general_codebooks) {
        int cell_of[15];
        for (int k = 1; k <= 15; ++k) cell_of[k - 1] = (int)floor(pseudo_angle(ctx->boundaries[0][k]) * 128.0);
        for (int cell = 0, before = 0; cell < 512; ++cell) {
            c.lut1[cell].thr = INFINITY;
            c.lut1[cell].count = (uint32_t)before;
            for (int k = 0; k < 15; ++k)
                if (cell_of[k] == cell) { c.lut1[cell].thr = (float)pseudo_angle(ctx->boundaries[0][k + 1]); ++before; }
        }
    }
    for (int k = 0; k < 16; ++k) {
        double t = ctx->centroids[0][k];
        c.cs1[k][0] = (float)cos(t);
        c.cs1[k][1] = (float)sin(t);
    }
    for (int l = 2; l <= 4; ++l)
        for (int k = 0; k < 4; ++k) {
            double t = ctx->centroids[l - 1][k];
            c.cs234[l - 2][k][0] = (float)cos(t);
            c.cs234[l - 2][k][1] = (float)sin(t);
        }
    /* The attention kernels' LDS image (layout: PQ_TAB_* in pq_common.h).  Entries are products of exact cosines and
       sines formed in double precision and rounded once. */
    auto f2u = [](float f) { uint32_t u; memcpy(&u, &f, 4); return u; };
    for (int t = 0; t < PQ_TAB_DWORDS; ++t) c.attn_tab[t] = 0u;
    for (int q = 0; q < 1024; ++q) { /* Q = c1' << 6 | c2 << 4 | c1 */
        const double t2 = ctx->centroids[1][(q >> 4) & 3], t1a = ctx->centroids[0][q & 15], t1b = ctx->centroids[0][q >> 6];
        c.attn_tab[PQ_TAB_TQ + 2 * q] = pack_h2(cos(t2) * cos(t1a), cos(t2) * sin(t1a));
        c.attn_tab[PQ_TAB_TQ + 2 * q + 1] = pack_h2(sin(t2) * cos(t1b), sin(t2) * sin(t1b));
    }
    for (int e = 0; e < 64; ++e) {
        {   /* e = c2 << 4 | c1 */
            const double t2 = ctx->centroids[1][e >> 4], t1 = ctx->centroids[0][e & 15];
            c.attn_tab[PQ_TAB_TQA + e] = pack_h2(cos(t2) * cos(t1), cos(t2) * sin(t1));
        }
        {   /* e = c1' << 2 | c2 */
            const double t2 = ctx->centroids[1][e & 3], t1 = ctx->centroids[0][e >> 2];
            c.attn_tab[PQ_TAB_TQB + e] = pack_h2(sin(t2) * cos(t1), sin(t2) * sin(t1));
        }
    }
    for (int b = 0; b < 64; ++b) {
        const double t4 = ctx->centroids[3][b >> 4], t3a = ctx->centroids[2][(b >> 2) & 3], t3b = ctx->centroids[2][b & 3];
        const double v[4] = {cos(t4) * cos(t3a), cos(t4) * sin(t3a), sin(t4) * cos(t3b), sin(t4) * sin(t3b)};
        for (int j = 0; j < 4; ++j) c.attn_tab[PQ_TAB_TBF + 4 * b + j] = f2u((float)v[j]);
        c.attn_tab[PQ_TAB_TBH + 2 * b] = pack_h2(v[0], v[1]);
        c.attn_tab[PQ_TAB_TBH + 2 * b + 1] = pack_h2(v[2], v[3]);
    }
    if (ctx->depth == 7)
        for (int l = 0; l < 3; ++l)
            for (int k = 0; k < 8; ++k)
                for (int h = 0; h < 2; ++h) c.attn_tab[PQ_TAB_UP + 16 * l + 2 * k + h] = f2u(c.up_cs[l][k][h]);
}

} // namespace

extern "C" const char *pq_status_string(pq_status s)
{
    switch (s) {
    case PQ_OK: return "PQ_OK";
    case PQ_EINVAL: return "PQ_EINVAL: invalid argument";
    case PQ_EUNSUPPORTED: return "PQ_EUNSUPPORTED: configuration not supported";
    case PQ_EALIGN: return "PQ_EALIGN: device pointer or stride not 16-byte aligned";
    case PQ_EHIP: return "PQ_EHIP: HIP runtime error or no device";
    case PQ_ENOMEM: return "PQ_ENOMEM: allocation failed or workspace too small";
    case PQ_ESCRATCH: return "PQ_ESCRATCH: the problem needs more than the static scratch buffer (pq_static_scratch_bytes)";
    case PQ_ENOTREADY: return "PQ_ENOTREADY: the context's constants are not on this device yet (call pq_prepare_device first)";
    }
    return "unknown pq_status";
}

namespace {

/* S = D H / sqrt(d): H the Sylvester Hadamard matrix H[i][j] = (-1)^popcount(i & j), D a diagonal of
   random signs (bit 63 of the counter-based generator at counter i), so y = x S flips the sign of
   coordinate i by D_i and then applies the Hadamard transform. */
void fill_randomised_hadamard(uint64_t seed, int d, double *S)
{
    const uint64_t sm = splitmix_finalise(seed ^ 0x48414441ULL);
    const double inv = 1.0 / sqrt((double)d);
    for (int i = 0; i < d; ++i) {
        const uint64_t bits = splitmix_finalise(sm + ((uint64_t)i + 1) * 0x9E3779B97F4A7C15ULL);
        const double di = (bits >> 63) ? -1.0 : 1.0;
        for (int j = 0; j < d; ++j) S[(size_t)i * d + j] = (__builtin_popcount((unsigned)(i & j)) & 1) ? -di * inv : di * inv;
    }
}

} // namespace

static pq_status init_context(pq_ctx **out, int d, uint64_t seed, const double *S_in, bool hadamard);

extern "C" pq_status pq_init_preconditioner(pq_ctx **out, int d, uint64_t seed, const double *S_in)
{
    return init_context(out, d, seed, S_in, false);
}

extern "C" pq_status pq_init_preconditioner_hadamard(pq_ctx **out, int d, uint64_t seed)
{
    return init_context(out, d, seed, nullptr, true);
}

static pq_status init_context(pq_ctx **out, int d, uint64_t seed, const double *S_in, bool hadamard)
{
    if (!out) return PQ_EINVAL;
    *out = nullptr;
    if (d != PQ_D) return PQ_EUNSUPPORTED;
    pq_ctx *ctx = new (std::nothrow) pq_ctx();
    if (!ctx) return PQ_ENOMEM;
    ctx->d = d;
    ctx->seed = seed;
    ctx->general_codebooks = false;
    ctx->depth = 4;
    if (S_in) {
        memcpy(ctx->S, S_in, sizeof(double) * d * d);
        for (int i = 0; i < d * d; ++i)
            if (!isfinite(ctx->S[i])) { delete ctx; return PQ_EINVAL; }
        if (!(orthogonality_defect(ctx->S, d) <= 1e-10)) { delete ctx; return PQ_EINVAL; }
    } else if (hadamard) {
        fill_randomised_hadamard(seed, d, ctx->S);
    } else {
        std::vector<double> G;
        fill_gaussian(seed, d, G);
        if (!orthonormalise_columns(G, d, ctx->S)) { delete ctx; return PQ_EINVAL; }
    }
    ctx->unit_entries = true;
    for (int i = 0; i < d * d; ++i)
        if (fabs(fabs(ctx->S[i]) * sqrt((double)d) - 1.0) > 1e-12) { ctx->unit_entries = false; break; }
    /* S = D H / sqrt(d) with the Sylvester H: row i is D_i = sign of S[i][0] times (-1)^popcount(i & j) */
    ctx->hadamard = PqHadamard{};
    if (ctx->unit_entries) {
        bool sylvester = true;
        for (int i = 0; i < d && sylvester; ++i)
            for (int j = 0; j < d; ++j) {
                const bool neg = ctx->S[(size_t)i * d + j] < 0.0, neg_row = ctx->S[(size_t)i * d] < 0.0;
                if (neg != (neg_row != ((__builtin_popcount((unsigned)(i & j)) & 1) != 0))) { sylvester = false; break; }
            }
        if (sylvester) {
            ctx->hadamard.on = 1u;
            for (int i = 0; i < d; ++i)
                if (ctx->S[(size_t)i * d] < 0.0) ctx->hadamard.neg[i >> 5] |= 1u << (i & 31);
        }
    }
    /* level 1: uniform density on [0, 2 pi): equal cells, centroids at their middles */
    for (int k = 0; k < 16; ++k) ctx->centroids[0][k] = (k + 0.5) * kPi / 8.0;
    for (int k = 0; k <= 16; ++k) ctx->boundaries[0][k] = k * kPi / 8.0;
    for (int l = 2; l <= 4; ++l) lloyd_max_level(l, ctx->centroids[l - 1], ctx->boundaries[l - 1]);
    build_tables(ctx);
    *out = ctx;
    return PQ_OK;
}

extern "C" int pq_preconditioner_structure(const pq_ctx *ctx)
{
    if (!ctx) return -1;
    return ctx->hadamard.on ? 2 : (ctx->unit_entries ? 1 : 0);
}

extern "C" pq_status pq_set_codebooks(pq_ctx *ctx, const double *cb)
{
    if (!ctx || !cb) return PQ_EINVAL;
    std::lock_guard<std::mutex> lock(ctx->mu);
    for (int i = 0; i < PQ_MAX_DEVICES; ++i)
        if (ctx->dev[i].ready) return PQ_EINVAL; /* tables already on a device: the context is in use */
    const int off[4] = {0, 16, 20, 24}, K[4] = {16, 4, 4, 4};
    const double hi[4] = {2.0 * kPi, kPi / 2.0, kPi / 2.0, kPi / 2.0};
    for (int l = 0; l < 4; ++l)
        for (int k = 0; k < K[l]; ++k) {
            const double t = cb[off[l] + k];
            if (!isfinite(t) || t < 0.0 || t >= hi[l]) return PQ_EINVAL;
            if (k > 0 && !(t > cb[off[l] + k - 1])) return PQ_EINVAL; /* strictly increasing */
        }
    /* level 1: at most one boundary per pseudo-angle cell (cells are 0.008-0.011 rad wide) */
    {
        int last = -1;
        for (int k = 1; k < 16; ++k) {
            const int cell = (int)floor(pseudo_angle(0.5 * (cb[k - 1] + cb[k])) * 128.0);
            if (cell <= last || cell > 511) return PQ_EUNSUPPORTED;
            last = cell;
        }
    }
    for (int l = 0; l < 4; ++l) {
        for (int k = 0; k < K[l]; ++k) ctx->centroids[l][k] = cb[off[l] + k];
        ctx->boundaries[l][0] = 0.0;
        ctx->boundaries[l][K[l]] = hi[l];
        for (int k = 1; k < K[l]; ++k) ctx->boundaries[l][k] = 0.5 * (ctx->centroids[l][k - 1] + ctx->centroids[l][k]);
    }
    ctx->general_codebooks = true;
    build_tables(ctx);
    return PQ_OK;
}

extern "C" pq_status pq_set_recursion_depth(pq_ctx *ctx, int depth, const int *upper_bits)
{
    if (!ctx) return PQ_EINVAL;
    if (depth != 4 && depth != 7) return PQ_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(ctx->mu);
    for (int i = 0; i < PQ_MAX_DEVICES; ++i)
        if (ctx->dev[i].ready) return PQ_EINVAL; /* tables already on a device: the context is in use */
    if (depth == 7) {
        if (!upper_bits) return PQ_EINVAL;
        for (int l = 0; l < 3; ++l)
            if (upper_bits[l] < 1 || upper_bits[l] > 3) return PQ_EINVAL;
        if (4 * upper_bits[0] + 2 * upper_bits[1] + upper_bits[2] > 16) return PQ_EUNSUPPORTED;
        for (int l = 0; l < 3; ++l) {
            ctx->upper_bits[l] = upper_bits[l];
            lloyd_max_level(5 + l, ctx->upper_centroids[l], ctx->upper_boundaries[l], 1 << upper_bits[l]);
        }
    }
    ctx->depth = depth;
    build_tables(ctx);
    return PQ_OK;
}

extern "C" pq_status pq_set_upper_codebooks(pq_ctx *ctx, const double *cbt)
{
    if (!ctx || !cbt) return PQ_EINVAL;
    std::lock_guard<std::mutex> lock(ctx->mu);
    if (ctx->depth != 7) return PQ_EINVAL;
    for (int i = 0; i < PQ_MAX_DEVICES; ++i)
        if (ctx->dev[i].ready) return PQ_EINVAL; /* tables already on a device: the context is in use */
    for (int l = 0; l < 3; ++l) {
        const int K = 1 << ctx->upper_bits[l];
        for (int k = 0; k < K; ++k) {
            const double t = cbt[8 * l + k];
            if (!isfinite(t) || t <= 0.0 || t >= kPi / 2.0) return PQ_EINVAL;
            if (k > 0 && !(t > cbt[8 * l + k - 1])) return PQ_EINVAL; /* strictly increasing */
        }
    }
    for (int l = 0; l < 3; ++l) {
        const int K = 1 << ctx->upper_bits[l];
        for (int k = 0; k < K; ++k) ctx->upper_centroids[l][k] = cbt[8 * l + k];
        ctx->upper_boundaries[l][0] = 0.0;
        ctx->upper_boundaries[l][K] = kPi / 2.0;
        for (int k = 1; k < K; ++k)
            ctx->upper_boundaries[l][k] = 0.5 * (ctx->upper_centroids[l][k - 1] + ctx->upper_centroids[l][k]);
    }
    build_tables(ctx);
    return PQ_OK;
}

extern "C" int pq_recursion_depth(const pq_ctx *ctx) { return ctx ? ctx->depth : 0; }

extern "C" int pq_radii_halves_per_tile(const pq_ctx *ctx)
{
    return !ctx ? 0 : (ctx->depth == 7 ? PQ_DEEP_RADII_HALVES : PQL_RADII);
}

extern "C" int pq_record_bytes(const pq_ctx *ctx)
{
    return !ctx ? 0 : (ctx->depth == 7 ? PQ_DEEP_RECORD_BYTES : PQ_RECORD_BYTES);
}

extern "C" pq_status pq_get_upper_codebook(const pq_ctx *ctx, int level, int *bits, double *centroids, double *boundaries)
{
    if (!ctx || level < 5 || level > 7) return PQ_EINVAL;
    if (ctx->depth != 7) return PQ_EINVAL;
    const int K = 1 << ctx->upper_bits[level - 5];
    if (bits) *bits = ctx->upper_bits[level - 5];
    if (centroids) memcpy(centroids, ctx->upper_centroids[level - 5], sizeof(double) * K);
    if (boundaries) memcpy(boundaries, ctx->upper_boundaries[level - 5], sizeof(double) * (K + 1));
    return PQ_OK;
}

extern "C" pq_status pq_get_preconditioner(const pq_ctx *ctx, double *S_out)
{
    if (!ctx || !S_out) return PQ_EINVAL;
    memcpy(S_out, ctx->S, sizeof(double) * PQ_D * PQ_D);
    return PQ_OK;
}

extern "C" pq_status pq_get_codebook(const pq_ctx *ctx, int level, double *centroids, double *boundaries)
{
    if (!ctx || level < 1 || level > 4) return PQ_EINVAL;
    int K = level == 1 ? 16 : 4;
    if (centroids) memcpy(centroids, ctx->centroids[level - 1], sizeof(double) * K);
    if (boundaries) memcpy(boundaries, ctx->boundaries[level - 1], sizeof(double) * (K + 1));
    return PQ_OK;
}

extern "C" void pq_destroy(pq_ctx *ctx)
{
    if (!ctx) return;
    int saved = -1;
    bool have_dev = hipGetDevice(&saved) == hipSuccess;
    for (int i = 0; i < PQ_MAX_DEVICES; ++i) {
        PqDeviceState &s = ctx->dev[i];
        if (!s.ready) continue;
        if (hipSetDevice(i) != hipSuccess) continue;
        (void)hipFree(s.consts);
        (void)hipFree(s.S_f32);
        (void)hipFree(s.St_f32);
        (void)hipFree(s.S_bf16x3);
    }
    if (have_dev) (void)hipSetDevice(saved);
    delete ctx;
}

pq_status pq_device_state(const pq_ctx *cctx, const PqDeviceState **out)
{
    pq_ctx *ctx = const_cast<pq_ctx *>(cctx);
    int dev = -1;
    PQ_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= PQ_MAX_DEVICES) return PQ_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(ctx->mu);
    PqDeviceState &s = ctx->dev[dev];
    if (!s.ready) {
        const int d = PQ_D;
        std::vector<float> Sf((size_t)d * d), Stf((size_t)d * d);
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < d; ++j) {
                Sf[(size_t)i * d + j] = (float)ctx->S[(size_t)i * d + j];
                Stf[(size_t)j * d + i] = (float)ctx->S[(size_t)i * d + j];
            }
        /* S = S1 + S2 + S3 with bf16 terms (24 significant bits in total), stored in
           the order the encode kernel's matrix-core A operand consumes them. */
        std::vector<uint16_t> sb((size_t)3 * PQ_SB_TERM_STRIDE);
        for (int rt = 0; rt < 4; ++rt)
            for (int ks = 0; ks < 8; ++ks)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e) {
                        int kg = lane >> 5, i = lane & 31;
                        /* k-step ks contracts input coordinates 8 ks .. 8 ks + 7 (lane half 0) and
                           64 + 8 ks .. (lane half 1): a lane of the kernel then reads one contiguous
                           half of its input row over the eight k-steps */
                        int row = 64 * kg + 8 * ks + e;
                        int col = 16 * (4 * ((i >> 2) & 1) + rt) + 4 * (i >> 3) + (i & 3);
                        double v = ctx->S[(size_t)row * d + col];
                        if (ctx->unit_entries) v = v < 0 ? -1.0 : 1.0; /* sqrt(d) * S, exact */
                        uint16_t t1 = to_bfloat16(v);
                        double r1 = v - from_bfloat16(t1);
                        uint16_t t2 = to_bfloat16(r1);
                        double r2 = r1 - from_bfloat16(t2);
                        uint16_t t3 = to_bfloat16(r2);
                        size_t at = ((((size_t)rt * 8 + ks) * 64 + lane) * 8 + e);
                        sb[at] = t1;
                        sb[PQ_SB_TERM_STRIDE + at] = t2;
                        sb[2 * (size_t)PQ_SB_TERM_STRIDE + at] = t3;
                    }
        PqDeviceState t;
        auto release = [&t]() { /* a failed set-up leaves nothing behind: the next call starts over */
            (void)hipFree(t.consts); (void)hipFree(t.S_f32); (void)hipFree(t.St_f32); (void)hipFree(t.S_bf16x3);
        };
        if (hipMalloc((void **)&t.consts, sizeof(PqDeviceConsts)) != hipSuccess ||
            hipMalloc((void **)&t.S_f32, Sf.size() * 4) != hipSuccess ||
            hipMalloc((void **)&t.St_f32, Stf.size() * 4) != hipSuccess ||
            hipMalloc((void **)&t.S_bf16x3, sb.size() * 2) != hipSuccess) {
            release();
            return PQ_ENOMEM;
        }
        if (hipMemcpy(t.consts, &ctx->host_consts, sizeof(PqDeviceConsts), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(t.S_f32, Sf.data(), Sf.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(t.St_f32, Stf.data(), Stf.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(t.S_bf16x3, sb.data(), sb.size() * 2, hipMemcpyHostToDevice) != hipSuccess) {
            release();
            return PQ_EHIP;
        }
        t.ready = true;
        s = t;
    }
    *out = &s;
    return PQ_OK;
}

bool pq_device_state_ready(const pq_ctx *cctx)
{
    pq_ctx *ctx = const_cast<pq_ctx *>(cctx);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= PQ_MAX_DEVICES) return false;
    std::lock_guard<std::mutex> lock(ctx->mu);
    return ctx->dev[dev].ready;
}

/* ---- optional kernel timing with HIP events on the launch stream ---- */
namespace {
struct Profiler {
    std::mutex mu;
    std::atomic<bool> on{false}; /* read without the lock on every launch */
    int cap = 0;
    std::vector<hipEvent_t> start[2], stop[2];
    int used[2] = {0, 0};
    int every = 1;            /* every `every`-th launch of a kernel is timed */
    int seen[2] = {0, 0};     /* launches since pq_profile_begin */
    bool timing_now[2] = {false, false};
} g_prof;
} // namespace

void pq_prof_before(int kind, hipStream_t s)
{
    if (!g_prof.on.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (!g_prof.on.load()) return;
    g_prof.timing_now[kind] = g_prof.used[kind] < g_prof.cap && (g_prof.seen[kind] % g_prof.every) == 0;
    g_prof.seen[kind] += 1;
    if (g_prof.timing_now[kind]) (void)hipEventRecord(g_prof.start[kind][g_prof.used[kind]], s);
}

void pq_prof_after(int kind, hipStream_t s)
{
    if (!g_prof.on.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.on.load() && g_prof.timing_now[kind]) {
        (void)hipEventRecord(g_prof.stop[kind][g_prof.used[kind]], s);
        g_prof.used[kind] += 1;
        g_prof.timing_now[kind] = false;
    }
}

extern "C" pq_status pq_profile_begin(int max_launches) { return pq_profile_begin_sampled(max_launches, 1); }

extern "C" pq_status pq_profile_begin_sampled(int max_launches, int every)
{
    if (max_launches <= 0 || max_launches > 65536 || every <= 0) return PQ_EINVAL;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.on) return PQ_EINVAL;
    for (int k = 0; k < 2; ++k) {
        while ((int)g_prof.start[k].size() < max_launches) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return PQ_EHIP;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return PQ_EHIP; }
            g_prof.start[k].push_back(a);
            g_prof.stop[k].push_back(b);
        }
        g_prof.used[k] = 0;
        g_prof.seen[k] = 0;
        g_prof.timing_now[k] = false;
    }
    g_prof.every = every;
    g_prof.cap = max_launches;
    g_prof.on = true;
    return PQ_OK;
}

extern "C" pq_status pq_profile_end(double *attn_ms, int *attn_launches, double *encode_ms, int *encode_launches)
{
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (!g_prof.on) return PQ_EINVAL;
    g_prof.on = false;
    double total[2] = {0.0, 0.0};
    for (int k = 0; k < 2; ++k)
        for (int i = 0; i < g_prof.used[k]; ++i) {
            float ms = 0.f;
            if (hipEventSynchronize(g_prof.stop[k][i]) != hipSuccess) return PQ_EHIP;
            if (hipEventElapsedTime(&ms, g_prof.start[k][i], g_prof.stop[k][i]) != hipSuccess) return PQ_EHIP;
            total[k] += ms;
        }
    if (attn_ms) *attn_ms = total[0];
    if (attn_launches) *attn_launches = g_prof.used[0];
    if (encode_ms) *encode_ms = total[1];
    if (encode_launches) *encode_launches = g_prof.used[1];
    return PQ_OK;
}
