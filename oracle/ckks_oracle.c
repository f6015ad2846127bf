/*
 * ckks_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU implementation of RNS-CKKS with hybrid
 * (digit) key switching: the scheme that sits below the HISA instructions of
 * the CHET paper (Fig. "Instructions of the HISA": encrypt, decrypt, encode,
 * decode, rotLeft/rotRight, add/sub, mul/mulPlain/mulScalar, divScalar,
 * mulNoRelin/relinearize) in its "RNS variant" reading (Sec. "HISA", Division
 * profile: the divisor is one coprime modulus of the ciphertext).
 *
 * Every modular product is (unsigned __int128) a*b % q.  No Barrett, no
 * Shoup, no Montgomery, no lazy reduction, no blocking, no fusion: each
 * function is the textbook definition of its step so that it can be checked
 * against the mathematics by eye.  Nothing here is shared with the GPU
 * library; only tests, the smoke check and the cpu_baseline leg of the
 * benchmark may load this file.
 *
 * Polynomials live in R_q = Z_q[X]/(X^N+1) as arrays of N uint64 residues in
 * [0,q).  "NTT form" means the vector (a(psi^(2*brv(i)+1)))_i, psi a
 * primitive 2N-th root of unity mod q and brv the bit reversal on log2 N bits.
 * Ciphertexts are kept in NTT form, layout [poly][limb][N].
 *
 * Pins (tests/test_oracle_*.py): NTT against the defining O(N^2) sum and
 * against schoolbook negacyclic convolution; PRNG against stored vectors;
 * the Gaussian table against its defining pmf; base conversion, mod-down and
 * rescale against big-integer identities; decrypt(encrypt) and rotation
 * against plaintext slot arithmetic; keys against their defining relation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

#define ORC_MAX_PRIMES 96

/* ------------------------------------------------------------------ */
/* modular arithmetic: the definition, nothing else                    */
/* ------------------------------------------------------------------ */
static u64 addmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + b) % q); }
static u64 submod(u64 a, u64 b, u64 q) { return (u64)(((u128)a + q - b) % q); }
static u64 mulmod(u64 a, u64 b, u64 q) { return (u64)(((u128)a * b) % q); }
static u64 negmod(u64 a, u64 q) { return a ? q - a : 0; }

static u64 powmod(u64 a, u64 e, u64 q) {
    u64 r = 1 % q;
    a %= q;
    while (e) {
        if (e & 1) r = mulmod(r, a, q);
        a = mulmod(a, a, q);
        e >>= 1;
    }
    return r;
}

/* inverse modulo a prime q by Fermat */
static u64 invmod(u64 a, u64 q) { return powmod(a, q - 2, q); }

/* signed integer -> residue in [0,q) */
static u64 reduce_i64(i64 v, u64 q) {
    if (v >= 0) return (u64)v % q;
    u64 m = (u64)(-(v + 1)) + 1; /* |v| without overflow */
    return negmod(m % q, q);
}

u64 orc_mulmod(u64 a, u64 b, u64 q) { return mulmod(a, b, q); }
u64 orc_powmod(u64 a, u64 e, u64 q) { return powmod(a, e, q); }

/* ------------------------------------------------------------------ */
/* primes and roots                                                    */
/* ------------------------------------------------------------------ */

/* Miller-Rabin with the first twelve primes as bases: exact below 2^64. */
int orc_is_prime(u64 n) {
    static const u64 bases[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return 0;
    for (int i = 0; i < 12; i++) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    u64 d = n - 1;
    int r = 0;
    while ((d & 1) == 0) { d >>= 1; r++; }
    for (int i = 0; i < 12; i++) {
        u64 x = powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int composite = 1;
        for (int j = 1; j < r; j++) {
            x = mulmod(x, x, n);
            if (x == n - 1) { composite = 0; break; }
        }
        if (composite) return 0;
    }
    return 1;
}

/*
 * A "b-bit NTT-friendly prime" is a prime p = 1 (mod 2N), p < 2^b.  Candidates
 * 2^b + 1 - t*2N for t = 1,2,...; the first prime not in used[0..n_used) wins.
 * Returns 0 when the candidates run out.
 */
u64 orc_next_prime(int bits, int log_n, const u64 *used, int n_used) {
    u64 two_n = (u64)2 << log_n;
    u64 c = ((u64)1 << bits) + 1;
    while (c > two_n) {
        c -= two_n;
        if (!orc_is_prime(c)) continue;
        int taken = 0;
        for (int i = 0; i < n_used; i++) taken |= (used[i] == c);
        if (!taken) return c;
    }
    return 0;
}

/* psi = x^((q-1)/2N) for the smallest x >= 2 that gives psi^N = -1 (mod q). */
u64 orc_find_psi(u64 q, int log_n) {
    u64 n = (u64)1 << log_n;
    for (u64 x = 2; x < q; x++) {
        u64 psi = powmod(x, (q - 1) / (2 * n), q);
        if (powmod(psi, n, q) == q - 1) return psi;
    }
    return 0;
}

static u64 bitrev(u64 x, int bits) {
    u64 r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}

/* ------------------------------------------------------------------ */
/* counter-based generator and samplers                                */
/* ------------------------------------------------------------------ */
#define RC1 0x6a09e667f3bcc909ULL
#define RC2 0xbb67ae8584caa73bULL
#define RC3 0x3c6ef372fe94f82bULL

static u64 mix64(u64 x) {
    x ^= x >> 32; x *= RC1;
    x ^= x >> 29; x *= RC2;
    x ^= x >> 32;
    return x;
}

/* kind: 1 secret, 2 encryption a, 3 encryption e, 4 key a, 5 key e */
u64 orc_rnd(u64 seed, u64 kind, u64 ctr, u64 idx) {
    u64 stream = ((kind << 56) | ctr) + 1;
    return mix64(mix64(seed + RC3 * stream) + RC3 * (idx + 1));
}

/* floor(2^63 * P(|X| <= k)), k = 0..18, X ~ pmf exp(-x^2 / (2*3.2^2)) on |x| <= 19 */
static const u64 GAUSS_CDT[19] = {
    1149872836518706973ULL, 3340023669317320718ULL, 5231742859181312982ULL,
    6713673040852152709ULL, 7766573333558595572ULL, 8445050410543775182ULL,
    8841576294031517592ULL, 9051758687454227207ULL, 9152802460441190481ULL,
    9196859083481262423ULL, 9214281214904026344ULL, 9220529772758650828ULL,
    9222562348483741346ULL, 9223162004373033245ULL, 9223322456656299389ULL,
    9223361395058736926ULL, 9223369965413244325ULL, 9223371676247247624ULL,
    9223371985993021523ULL};

void orc_gauss_table(u64 *out19) { memcpy(out19, GAUSS_CDT, sizeof GAUSS_CDT); }

/* The same table for another sigma (optional parameter of the scheme's initialisation): tail cut at
 * K = floor(6 sigma) <= ORC_MAX_CDT, out[k] = floor(2^63 * P(|X| <= k)) for k = 0..K-1, pmf proportional to
 * exp(-x^2 / (2 sigma^2)) on |x| <= K.  sigma = 3.2 gives the table above (typed in from an 80-digit
 * computation); any other is computed here in long double: weights w_x = expl(-x^2 / (2 sigma^2)), running sums
 * c_0 = w_0, c_k = c_{k-1} + 2 w_k, total = c_K, entry k = floorl(2^63 * (c_k / total)) -- within a few units of
 * 2^-63 of the exact value.  Returns K, or 0 for a sigma outside (0.2, ORC_MAX_CDT / 6]. */
#define ORC_MAX_CDT 60
int orc_gauss_table_for(double sigma, u64 *out) {
    if (sigma == 3.2) { memcpy(out, GAUSS_CDT, sizeof GAUSS_CDT); return 19; }
    if (!(sigma > 0.2) || sigma * 6.0 > (double)ORC_MAX_CDT) return 0;
    int K = (int)floor(6.0 * sigma);
    long double two_s2 = 2.0L * (long double)sigma * (long double)sigma;
    long double c[ORC_MAX_CDT + 1];
    for (int x = 0; x <= K; x++) {
        long double w = expl(-((long double)x * (long double)x) / two_s2);
        c[x] = x == 0 ? w : c[x - 1] + 2.0L * w;
    }
    for (int k = 0; k < K; k++) {
        long double v = floorl(ldexpl(c[k] / c[K], 63));
        out[k] = v >= 9223372036854775807.0L ? 9223372036854775807ULL : (u64)v;
    }
    return K;
}

/* one discrete Gaussian integer from one 64-bit word */
i64 orc_gauss_from_word(u64 u) {
    int negative = (int)(u & 1);
    u64 v = u >> 1;
    i64 mag = 0;
    for (int k = 0; k < 19; k++) mag += (v >= GAUSS_CDT[k]);
    return negative ? -mag : mag;
}

/* one ternary value from one word: 0 -> 0, 1 -> +1, 2 -> -1 */
i64 orc_ternary_from_word(u64 u) {
    u64 t = u % 3;
    return t == 0 ? 0 : (t == 1 ? 1 : -1);
}

/* ------------------------------------------------------------------ */
/* context                                                             */
/* ------------------------------------------------------------------ */
typedef struct {
    int log_n;
    u64 n;          /* ring degree N */
    int L;          /* ciphertext primes q_0..q_{L-1} */
    int K;          /* special primes p_0..p_{K-1}; K = alpha */
    int dnum;
    int alpha;      /* primes per digit = ceil(L/dnum) */
    u64 seed;
    int noise;      /* 0: all error polynomials are zero; 1: discrete Gaussian with the table below */
    u64 cdt[ORC_MAX_CDT];      /* floor(2^63 P(|X| <= k)) of the context's sigma */
    int cdt_n;
    u64 mod[ORC_MAX_PRIMES];   /* q_0..q_{L-1}, p_0..p_{K-1} */
    u64 psi[ORC_MAX_PRIMES];
    u64 n_inv[ORC_MAX_PRIMES];
    u64 *psi_brv[ORC_MAX_PRIMES];      /* psi^brv(i) */
    u64 *psi_inv_brv[ORC_MAX_PRIMES];  /* psi^-brv(i) */
    i64 *s_coef;    /* ternary secret, coefficient form, N entries */
    u64 *s_ntt;     /* secret in NTT form over all L+K primes */
} orc_ctx;

void orc_destroy(orc_ctx *c) {
    if (!c) return;
    for (int i = 0; i < ORC_MAX_PRIMES; i++) { free(c->psi_brv[i]); free(c->psi_inv_brv[i]); }
    free(c->s_coef);
    free(c->s_ntt);
    free(c);
}

void orc_ntt(const orc_ctx *c, int prime, u64 *a);
void orc_intt(const orc_ctx *c, int prime, u64 *a);

/*
 * Parameters: log_n; num_q primes of q_bits[i] bits; dnum digits; alpha =
 * ceil(num_q/dnum) special primes of special_bits bits, requested after the
 * q_i in order.  The ternary secret s is drawn here (kind 1, ctr 0, idx =
 * coefficient).
 */
static i64 gauss_from_table(const u64 *cdt, int cdt_n, u64 u) {
    int negative = (int)(u & 1);
    u64 v = u >> 1;
    i64 mag = 0;
    for (int k = 0; k < cdt_n; k++) mag += (v >= cdt[k]);
    return negative ? -mag : mag;
}

/* secret_kind 0: every coefficient uniform in {-1, 0, 1}.  secret_kind 1: exactly h non-zero coefficients (the
 * sparse secrets of HEAAN): a partial Fisher-Yates shuffle of the positions 0..N-1 -- step i = 0..h-1 draws the word
 * u = rnd(seed, 1, 0, i), exchanges position i of the permutation with position i + (u >> 1) mod (N - i), and the
 * coefficient now named by position i becomes -1 if the low bit of u is set, +1 otherwise. */
orc_ctx *orc_create_ex(int log_n, int num_q, const int *q_bits, int dnum, int special_bits,
                       u64 seed, int noise, double sigma, int secret_kind, int h);

orc_ctx *orc_create(int log_n, int num_q, const int *q_bits, int dnum, int special_bits,
                    u64 seed, int noise) {
    return orc_create_ex(log_n, num_q, q_bits, dnum, special_bits, seed, noise, 3.2, 0, 0);
}

orc_ctx *orc_create_ex(int log_n, int num_q, const int *q_bits, int dnum, int special_bits,
                       u64 seed, int noise, double sigma, int secret_kind, int h) {
    if (log_n < 1 || log_n > 17 || num_q < 1 || dnum < 1 || dnum > num_q) return NULL;
    if (secret_kind != 0 && secret_kind != 1) return NULL;
    if (secret_kind == 1 && (h < 1 || (u64)h > ((u64)1 << log_n))) return NULL;
    int alpha = (num_q + dnum - 1) / dnum;
    if (num_q + alpha > ORC_MAX_PRIMES) return NULL;
    orc_ctx *c = calloc(1, sizeof *c);
    c->log_n = log_n; c->n = (u64)1 << log_n;
    c->L = num_q; c->K = alpha; c->dnum = dnum; c->alpha = alpha;
    c->seed = seed; c->noise = noise;
    c->cdt_n = orc_gauss_table_for(sigma, c->cdt);
    if (!c->cdt_n) { free(c); return NULL; }
    int total = num_q + alpha;
    for (int i = 0; i < total; i++) {
        int bits = i < num_q ? q_bits[i] : special_bits;
        if (bits < log_n + 2 || bits > 60) { orc_destroy(c); return NULL; }
        c->mod[i] = orc_next_prime(bits, log_n, c->mod, i);
        if (!c->mod[i]) { orc_destroy(c); return NULL; }
        u64 q = c->mod[i];
        c->psi[i] = orc_find_psi(q, log_n);
        c->n_inv[i] = invmod(c->n % q, q);
        c->psi_brv[i] = malloc(c->n * sizeof(u64));
        c->psi_inv_brv[i] = malloc(c->n * sizeof(u64));
        u64 psi_inv = invmod(c->psi[i], q);
        for (u64 x = 0; x < c->n; x++) {
            u64 e = bitrev(x, log_n);
            c->psi_brv[i][x] = powmod(c->psi[i], e, q);
            c->psi_inv_brv[i][x] = powmod(psi_inv, e, q);
        }
    }
    c->s_coef = malloc(c->n * sizeof(i64));
    c->s_ntt = malloc((size_t)total * c->n * sizeof(u64));
    if (secret_kind == 0) {
        for (u64 j = 0; j < c->n; j++) c->s_coef[j] = orc_ternary_from_word(orc_rnd(seed, 1, 0, j));
    } else {
        u64 *perm = malloc(c->n * sizeof(u64));
        for (u64 j = 0; j < c->n; j++) { perm[j] = j; c->s_coef[j] = 0; }
        for (u64 i = 0; i < (u64)h; i++) {
            u64 u = orc_rnd(seed, 1, 0, i);
            u64 j = i + (u >> 1) % (c->n - i);
            u64 t = perm[i]; perm[i] = perm[j]; perm[j] = t;
            c->s_coef[perm[i]] = (u & 1) ? -1 : 1;
        }
        free(perm);
    }
    for (int i = 0; i < total; i++) {
        u64 *dst = c->s_ntt + (size_t)i * c->n;
        for (u64 j = 0; j < c->n; j++) dst[j] = reduce_i64(c->s_coef[j], c->mod[i]);
        orc_ntt(c, i, dst);
    }
    return c;
}

int orc_num_primes(const orc_ctx *c) { return c->L + c->K; }
int orc_num_special(const orc_ctx *c) { return c->K; }
int orc_alpha(const orc_ctx *c) { return c->alpha; }
void orc_get_primes(const orc_ctx *c, u64 *out) { memcpy(out, c->mod, (size_t)(c->L + c->K) * sizeof(u64)); }
void orc_get_psi(const orc_ctx *c, u64 *out) { memcpy(out, c->psi, (size_t)(c->L + c->K) * sizeof(u64)); }
void orc_get_secret_coef(const orc_ctx *c, i64 *out) { memcpy(out, c->s_coef, c->n * sizeof(i64)); }

/* ------------------------------------------------------------------ */
/* negacyclic NTT                                                      */
/* ------------------------------------------------------------------ */

/*
 * Forward transform, in place: natural-order coefficients in, a(psi^(2*brv(i)+1))
 * out.  Decimation in time with the psi-twist merged into the butterflies: at
 * the level with m blocks, block i multiplies its lower half by psi^brv(m+i).
 */
void orc_ntt(const orc_ctx *c, int prime, u64 *a) {
    u64 q = c->mod[prime];
    const u64 *w = c->psi_brv[prime];
    u64 t = c->n;
    for (u64 m = 1; m < c->n; m <<= 1) {
        t >>= 1;
        for (u64 i = 0; i < m; i++) {
            u64 s = w[m + i];
            for (u64 j = 2 * i * t; j < 2 * i * t + t; j++) {
                u64 u = a[j];
                u64 v = mulmod(a[j + t], s, q);
                a[j] = addmod(u, v, q);
                a[j + t] = submod(u, v, q);
            }
        }
    }
}

/* Inverse transform, in place: the levels of orc_ntt undone in reverse, then 1/N. */
void orc_intt(const orc_ctx *c, int prime, u64 *a) {
    u64 q = c->mod[prime];
    const u64 *w = c->psi_inv_brv[prime];
    u64 t = 1;
    for (u64 m = c->n >> 1; m >= 1; m >>= 1) {
        for (u64 i = 0; i < m; i++) {
            u64 s = w[m + i];
            for (u64 j = 2 * i * t; j < 2 * i * t + t; j++) {
                u64 u = a[j];
                u64 v = a[j + t];
                a[j] = addmod(u, v, q);
                a[j + t] = mulmod(submod(u, v, q), s, q);
            }
        }
        t <<= 1;
    }
    for (u64 j = 0; j < c->n; j++) a[j] = mulmod(a[j], c->n_inv[prime], q);
}

/* ------------------------------------------------------------------ */
/* sampling of polynomials                                             */
/* ------------------------------------------------------------------ */

/* uniform polynomial, COEFFICIENT form: coefficient j mod prime i is
 * rnd(seed, kind, ctr, i*N + j) mod q_i */
void orc_sample_uniform(const orc_ctx *c, u64 kind, u64 ctr, int prime, u64 *out) {
    u64 q = c->mod[prime];
    for (u64 j = 0; j < c->n; j++) out[j] = orc_rnd(c->seed, kind, ctr, (u64)prime * c->n + j) % q;
}

/* error polynomial as signed integers (all zero when noise is off) */
void orc_sample_error(const orc_ctx *c, u64 kind, u64 ctr, i64 *out) {
    for (u64 j = 0; j < c->n; j++)
        out[j] = c->noise ? gauss_from_table(c->cdt, c->cdt_n, orc_rnd(c->seed, kind, ctr, j)) : 0;
}

/* signed coefficient vector -> NTT form modulo prime i */
void orc_signed_to_ntt(const orc_ctx *c, const i64 *coef, int prime, u64 *out) {
    for (u64 j = 0; j < c->n; j++) out[j] = reduce_i64(coef[j], c->mod[prime]);
    orc_ntt(c, prime, out);
}

/* ------------------------------------------------------------------ */
/* encoding (Sec. "HEAAN": N/2 complex slots, rounding at encode)      */
/* ------------------------------------------------------------------ */

/*
 * Slot j sits at the root zeta_j = exp(i*pi*5^j/N).  The real polynomial that
 * takes the values z_j there (and conj z_j at the conjugate roots) has
 * coefficients (2/N) Re sum_j z_j zeta_j^-k; encode scales by `scale` and
 * rounds half away from zero.  Direct O(N*n) sum in long double.  Missing
 * slots (count < N/2) are zero.  im may be NULL.
 */
void orc_encode(int log_n, const double *re, const double *im, u64 count, double scale, i64 *coef) {
    u64 n_ring = (u64)1 << log_n, slots = n_ring / 2, two_n = 2 * n_ring;
    long double *cs = malloc(two_n * sizeof(long double));
    long double *sn = malloc(two_n * sizeof(long double));
    const long double pi = 3.14159265358979323846264338327950288L;
    for (u64 t = 0; t < two_n; t++) {
        cs[t] = cosl(pi * (long double)t / (long double)n_ring);
        sn[t] = sinl(pi * (long double)t / (long double)n_ring);
    }
    if (count > slots) count = slots;
    for (u64 k = 0; k < n_ring; k++) {
        long double acc = 0.0L;
        u64 g = 1; /* 5^j mod 2N */
        for (u64 j = 0; j < count; j++) {
            u64 e = (g * k) % two_n; /* zeta_j^k = exp(i*pi*e/N) */
            long double zr = re[j], zi = im ? im[j] : 0.0;
            /* Re( z * conj(zeta_j^k) ) */
            acc += zr * cs[e] + zi * sn[e];
            g = (g * 5) % two_n;
        }
        long double v = acc * (2.0L * (long double)scale / (long double)n_ring);
        coef[k] = (i64)roundl(v);
    }
    free(cs); free(sn);
}

/*
 * Decode: z_j = (1/scale) sum_k m_k zeta_j^k with the real (centred integer)
 * coefficients m_k given as hi[k] + lo[k], two doubles, so that integers
 * beyond 2^53 keep their low bits.  Direct O(N*n) sum in long double.
 */
void orc_decode(int log_n, const double *hi, const double *lo, u64 count, double scale,
                double *re, double *im) {
    u64 n_ring = (u64)1 << log_n, slots = n_ring / 2, two_n = 2 * n_ring;
    long double *cs = malloc(two_n * sizeof(long double));
    long double *sn = malloc(two_n * sizeof(long double));
    const long double pi = 3.14159265358979323846264338327950288L;
    for (u64 t = 0; t < two_n; t++) {
        cs[t] = cosl(pi * (long double)t / (long double)n_ring);
        sn[t] = sinl(pi * (long double)t / (long double)n_ring);
    }
    if (count > slots) count = slots;
    u64 g = 1;
    for (u64 j = 0; j < count; j++) {
        long double ar = 0.0L, ai = 0.0L;
        for (u64 k = 0; k < n_ring; k++) {
            u64 e = (g * k) % two_n;
            long double m = (long double)hi[k] + (long double)lo[k];
            ar += m * cs[e];
            ai += m * sn[e];
        }
        re[j] = (double)(ar / (long double)scale);
        if (im) im[j] = (double)(ai / (long double)scale);
        g = (g * 5) % two_n;
    }
    free(cs); free(sn);
}

/* ------------------------------------------------------------------ */
/* encryption profile                                                  */
/* ------------------------------------------------------------------ */

/*
 * Symmetric encryption of a plaintext given in NTT form on primes q_0..q_{l-1}:
 * c1 = a (uniform, kind 2, counter ctr), c0 = -a*s + e + m (e: kind 3, same ctr).
 * ct layout [2][l][N], NTT form.
 */
void orc_encrypt(const orc_ctx *c, const u64 *pt, int l, u64 ctr, u64 *ct) {
    u64 n = c->n;
    i64 *e = malloc(n * sizeof(i64));
    u64 *e_ntt = malloc(n * sizeof(u64));
    orc_sample_error(c, 3, ctr, e);
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        u64 *c0 = ct + (size_t)i * n, *c1 = ct + (size_t)(l + i) * n;
        const u64 *s = c->s_ntt + (size_t)i * n;
        orc_sample_uniform(c, 2, ctr, i, c1);
        orc_ntt(c, i, c1);
        orc_signed_to_ntt(c, e, i, e_ntt);
        for (u64 j = 0; j < n; j++) {
            u64 as = mulmod(c1[j], s[j], q);
            c0[j] = addmod(addmod(negmod(as, q), e_ntt[j], q), pt[(size_t)i * n + j], q);
        }
    }
    free(e); free(e_ntt);
}

/* m' = c0 + c1*s (+ c2*s^2); ct [polys][l][N] -> pt [l][N], both NTT form */
void orc_decrypt(const orc_ctx *c, const u64 *ct, int polys, int l, u64 *pt) {
    u64 n = c->n;
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        const u64 *s = c->s_ntt + (size_t)i * n;
        for (u64 j = 0; j < n; j++) {
            u64 acc = ct[(size_t)i * n + j];
            u64 sp = s[j];
            for (int p = 1; p < polys; p++) {
                acc = addmod(acc, mulmod(ct[((size_t)p * l + i) * n + j], sp, q), q);
                sp = mulmod(sp, s[j], q);
            }
            pt[(size_t)i * n + j] = acc;
        }
    }
}

/* NTT form <-> coefficient form of `count` consecutive limb-polynomials whose
 * primes are first_prime, first_prime+1, ... repeated with period l */
void orc_to_coeff(const orc_ctx *c, u64 *x, int polys, int l) {
    for (int p = 0; p < polys; p++)
        for (int i = 0; i < l; i++) orc_intt(c, i, x + ((size_t)p * l + i) * c->n);
}
void orc_to_ntt(const orc_ctx *c, u64 *x, int polys, int l) {
    for (int p = 0; p < polys; p++)
        for (int i = 0; i < l; i++) orc_ntt(c, i, x + ((size_t)p * l + i) * c->n);
}

/* ------------------------------------------------------------------ */
/* limb-wise arithmetic (add, sub, mulPlain, mulScalar, mulNoRelin)    */
/* ------------------------------------------------------------------ */

/* out = a + b or a - b over polys*l limb-polynomials (equal shapes) */
void orc_add(const orc_ctx *c, const u64 *a, const u64 *b, int polys, int l, int subtract, u64 *out) {
    u64 n = c->n;
    for (int p = 0; p < polys; p++)
        for (int i = 0; i < l; i++) {
            u64 q = c->mod[i];
            size_t o = ((size_t)p * l + i) * n;
            for (u64 j = 0; j < n; j++)
                out[o + j] = subtract ? submod(a[o + j], b[o + j], q) : addmod(a[o + j], b[o + j], q);
        }
}

/* out = ct with pt added to (or subtracted from) its first polynomial */
void orc_add_plain(const orc_ctx *c, const u64 *ct, const u64 *pt, int polys, int l, int subtract, u64 *out) {
    u64 n = c->n;
    if (out != ct) memcpy(out, ct, (size_t)polys * l * n * sizeof(u64));
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        size_t o = (size_t)i * n;
        for (u64 j = 0; j < n; j++)
            out[o + j] = subtract ? submod(ct[o + j], pt[o + j], q) : addmod(ct[o + j], pt[o + j], q);
    }
}

/*
 * Adds the integer V (given modulo each q_i in v_mod[i]) to the constant
 * coefficient of the first polynomial; in NTT form the constant polynomial V
 * is V at every evaluation point.
 */
void orc_add_const(const orc_ctx *c, const u64 *ct, const u64 *v_mod, int polys, int l, int subtract, u64 *out) {
    u64 n = c->n;
    if (out != ct) memcpy(out, ct, (size_t)polys * l * n * sizeof(u64));
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        size_t o = (size_t)i * n;
        for (u64 j = 0; j < n; j++)
            out[o + j] = subtract ? submod(ct[o + j], v_mod[i], q) : addmod(ct[o + j], v_mod[i], q);
    }
}

/* every polynomial of ct times the plaintext, slot-wise in NTT form */
void orc_mul_plain(const orc_ctx *c, const u64 *ct, const u64 *pt, int polys, int l, u64 *out) {
    u64 n = c->n;
    for (int p = 0; p < polys; p++)
        for (int i = 0; i < l; i++) {
            u64 q = c->mod[i];
            size_t o = ((size_t)p * l + i) * n, po = (size_t)i * n;
            for (u64 j = 0; j < n; j++) out[o + j] = mulmod(ct[o + j], pt[po + j], q);
        }
}

/* every residue times the integer x given modulo each q_i */
void orc_mul_const(const orc_ctx *c, const u64 *ct, const u64 *x_mod, int polys, int l, u64 *out) {
    u64 n = c->n;
    for (int p = 0; p < polys; p++)
        for (int i = 0; i < l; i++) {
            u64 q = c->mod[i];
            size_t o = ((size_t)p * l + i) * n;
            for (u64 j = 0; j < n; j++) out[o + j] = mulmod(ct[o + j], x_mod[i], q);
        }
}

/* (a0,a1) x (b0,b1) -> (a0 b0, a0 b1 + a1 b0, a1 b1), layout [3][l][N] */
void orc_mul_no_relin(const orc_ctx *c, const u64 *a, const u64 *b, int l, u64 *out) {
    u64 n = c->n;
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        const u64 *a0 = a + (size_t)i * n, *a1 = a + (size_t)(l + i) * n;
        const u64 *b0 = b + (size_t)i * n, *b1 = b + (size_t)(l + i) * n;
        u64 *d0 = out + (size_t)i * n, *d1 = out + (size_t)(l + i) * n, *d2 = out + (size_t)(2 * l + i) * n;
        for (u64 j = 0; j < n; j++) {
            u64 x0 = mulmod(a0[j], b0[j], q);
            u64 x1 = addmod(mulmod(a0[j], b1[j], q), mulmod(a1[j], b0[j], q), q);
            u64 x2 = mulmod(a1[j], b1[j], q);
            d0[j] = x0; d1[j] = x1; d2[j] = x2;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Galois automorphism X -> X^g                                        */
/* ------------------------------------------------------------------ */

/* coefficient form, one limb: coefficient i moves to i*g mod 2N, negated if it lands in [N,2N) */
void orc_automorph_coeff(const orc_ctx *c, const u64 *a, u64 g, int prime, u64 *out) {
    u64 n = c->n, q = c->mod[prime];
    for (u64 i = 0; i < n; i++) {
        u64 t = (i * g) % (2 * n);
        if (t < n) out[t] = a[i];
        else out[t - n] = negmod(a[i], q);
    }
}

/* galois element of a left rotation by r slots: 5^r mod 2N */
u64 orc_galois_elt(int log_n, u64 r) {
    u64 two_n = (u64)2 << log_n, g = 1;
    r %= (two_n / 4);
    for (u64 i = 0; i < r; i++) g = (g * 5) % two_n;
    return g;
}

/* NTT-form limbs [l][N] -> sigma_g of them, by way of coefficient form */
void orc_automorph_ntt(const orc_ctx *c, const u64 *a, u64 g, int first_prime, int l, u64 *out) {
    u64 n = c->n;
    u64 *tmp = malloc(n * sizeof(u64));
    for (int i = 0; i < l; i++) {
        memcpy(tmp, a + (size_t)i * n, n * sizeof(u64));
        orc_intt(c, first_prime + i, tmp);
        orc_automorph_coeff(c, tmp, g, first_prime + i, out + (size_t)i * n);
        orc_ntt(c, first_prime + i, out + (size_t)i * n);
    }
    free(tmp);
}

/* ------------------------------------------------------------------ */
/* fast base conversion                                                */
/* ------------------------------------------------------------------ */

/*
 * x given by residues x[i][.] modulo the primes src[0..a) (indices into
 * c->mod, product D) is carried to the prime t = mod[dst]:
 *     y_i = x_i * (D/c_i)^-1 mod c_i, taken as the centred representative
 *           (y_i - c_i when y_i > floor(c_i/2)),
 *     out = sum_i y_i * (D/c_i)  mod t.
 * The integer sum_i y_i (D/c_i) equals x + u*D for the centred x and some
 * |u| <= a/2; that multiple of D is NOT removed (the fast, approximate
 * conversion).  Coefficient form on both sides.
 */
void orc_base_conv(const orc_ctx *c, const u64 *const *x, const int *src, int a, int dst, u64 *out) {
    u64 n = c->n, t = c->mod[dst];
    u64 inv_hat[ORC_MAX_PRIMES], hat_t[ORC_MAX_PRIMES];
    for (int i = 0; i < a; i++) {
        u64 ci = c->mod[src[i]];
        u64 hat_ci = 1 % ci, hat = 1 % t;
        for (int m = 0; m < a; m++) {
            if (m == i) continue;
            hat_ci = mulmod(hat_ci, c->mod[src[m]] % ci, ci);
            hat = mulmod(hat, c->mod[src[m]] % t, t);
        }
        inv_hat[i] = invmod(hat_ci, ci);
        hat_t[i] = hat;
    }
    for (u64 j = 0; j < n; j++) {
        u64 acc = 0;
        for (int i = 0; i < a; i++) {
            u64 ci = c->mod[src[i]];
            u64 y = mulmod(x[i][j], inv_hat[i], ci);
            u64 term = mulmod(y % t, hat_t[i], t);
            if (y > ci / 2) /* centred y_i = y - c_i: subtract c_i * (D/c_i) = D as well */
                term = submod(term, mulmod(ci % t, hat_t[i], t), t);
            acc = addmod(acc, term, t);
        }
        out[j] = acc;
    }
}

/* ------------------------------------------------------------------ */
/* evaluation keys and hybrid key switching                            */
/* ------------------------------------------------------------------ */

/*
 * Switching key towards the secret s' (given in NTT form over all L+K primes):
 * for digit j (primes q_{j*alpha} .. q_{min((j+1)alpha,L)-1}):
 *   a_j uniform over all L+K primes   (kind 4, ctr = (key_id<<8)|j)
 *   e_j one error polynomial          (kind 5, same ctr)
 *   b_j[i] = -a_j[i]*s + e_j + [i in digit j] * (P mod q_i) * s'     (i < L)
 *   b_j[i] = -a_j[i]*s + e_j                                        (special i)
 * with P the product of the special primes.  Layout [dnum][2][L+K][N], b then
 * a, NTT form.
 */
void orc_gen_switch_key(const orc_ctx *c, u64 key_id, const u64 *s_target, u64 *key) {
    u64 n = c->n;
    int total = c->L + c->K;
    i64 *e = malloc(n * sizeof(i64));
    u64 *e_ntt = malloc(n * sizeof(u64));
    for (int j = 0; j < c->dnum; j++) {
        u64 ctr = (key_id << 8) | (u64)j;
        orc_sample_error(c, 5, ctr, e);
        for (int i = 0; i < total; i++) {
            u64 q = c->mod[i];
            u64 *b = key + (((size_t)j * 2 + 0) * total + i) * n;
            u64 *a = key + (((size_t)j * 2 + 1) * total + i) * n;
            const u64 *s = c->s_ntt + (size_t)i * n;
            orc_sample_uniform(c, 4, ctr, i, a);
            orc_ntt(c, i, a);
            orc_signed_to_ntt(c, e, i, e_ntt);
            int in_digit = i < c->L && i / c->alpha == j;
            u64 p_mod = 1 % q;
            for (int m = 0; m < c->K; m++) p_mod = mulmod(p_mod, c->mod[c->L + m] % q, q);
            for (u64 x = 0; x < n; x++) {
                u64 v = addmod(negmod(mulmod(a[x], s[x], q), q), e_ntt[x], q);
                if (in_digit) v = addmod(v, mulmod(p_mod, s_target[(size_t)i * n + x], q), q);
                b[x] = v;
            }
        }
    }
    free(e); free(e_ntt);
}

/* s^2 in NTT form over all primes (target of the relinearisation key) */
void orc_secret_squared(const orc_ctx *c, u64 *out) {
    u64 n = c->n;
    for (int i = 0; i < c->L + c->K; i++)
        for (u64 j = 0; j < n; j++) {
            u64 s = c->s_ntt[(size_t)i * n + j];
            out[(size_t)i * n + j] = mulmod(s, s, c->mod[i]);
        }
}

/* sigma_g(s) in NTT form over all primes (target of the rotation key for g) */
void orc_secret_automorph(const orc_ctx *c, u64 g, u64 *out) {
    orc_automorph_ntt(c, c->s_ntt, g, 0, c->L + c->K, out);
}

/*
 * Mod-down of one accumulator: acc has l limbs modulo q_0..q_{l-1} followed by
 * K limbs modulo the special primes, NTT form.  The special limbs go to
 * coefficient form, are base-converted to each q_i (centred, so the division rounds), come
 * back to NTT form, and out[i] = (acc[i] - conv_i) * P^-1 mod q_i.
 */
void orc_mod_down(const orc_ctx *c, const u64 *acc, int l, u64 *out) {
    u64 n = c->n;
    u64 *sp = malloc((size_t)c->K * n * sizeof(u64));
    u64 *conv = malloc(n * sizeof(u64));
    const u64 *rows[ORC_MAX_PRIMES];
    int src[ORC_MAX_PRIMES];
    for (int m = 0; m < c->K; m++) {
        memcpy(sp + (size_t)m * n, acc + (size_t)(l + m) * n, n * sizeof(u64));
        orc_intt(c, c->L + m, sp + (size_t)m * n);
        rows[m] = sp + (size_t)m * n;
        src[m] = c->L + m;
    }
    for (int i = 0; i < l; i++) {
        u64 q = c->mod[i];
        orc_base_conv(c, rows, src, c->K, i, conv);
        orc_ntt(c, i, conv);
        u64 p_mod = 1 % q;
        for (int m = 0; m < c->K; m++) p_mod = mulmod(p_mod, c->mod[c->L + m] % q, q);
        u64 p_inv = invmod(p_mod, q);
        for (u64 j = 0; j < n; j++)
            out[(size_t)i * n + j] = mulmod(submod(acc[(size_t)i * n + j], conv[j], q), p_inv, q);
    }
    free(sp); free(conv);
}

/*
 * Mod-down and rescale in one division: the accumulator is divided by q_{l-1} * P instead of P, the limb of q_{l-1}
 * joining the special limbs as a source of the base conversion; out has l - 1 limbs,
 * out[i] = (acc[i] - conv_i) * (q_{l-1} P)^-1 mod q_i with conv the centred conversion of acc mod q_{l-1} P.
 */
void orc_mod_down_rescale(const orc_ctx *c, const u64 *acc, int l, u64 *out) {
    u64 n = c->n;
    int a = c->K + 1;
    u64 *sp = malloc((size_t)a * n * sizeof(u64));
    u64 *conv = malloc(n * sizeof(u64));
    const u64 *rows[ORC_MAX_PRIMES];
    int src[ORC_MAX_PRIMES];
    for (int m = 0; m < a; m++) {
        int pos = l - 1 + m, prime = m == 0 ? l - 1 : c->L + m - 1;
        memcpy(sp + (size_t)m * n, acc + (size_t)pos * n, n * sizeof(u64));
        orc_intt(c, prime, sp + (size_t)m * n);
        rows[m] = sp + (size_t)m * n;
        src[m] = prime;
    }
    for (int i = 0; i < l - 1; i++) {
        u64 q = c->mod[i];
        orc_base_conv(c, rows, src, a, i, conv);
        orc_ntt(c, i, conv);
        u64 d_mod = 1 % q;
        for (int m = 0; m < a; m++) d_mod = mulmod(d_mod, c->mod[src[m]] % q, q);
        u64 d_inv = invmod(d_mod, q);
        for (u64 j = 0; j < n; j++)
            out[(size_t)i * n + j] = mulmod(submod(acc[(size_t)i * n + j], conv[j], q), d_inv, q);
    }
    free(sp); free(conv);
}

/*
 * Hybrid key switch of one polynomial d (l limbs, NTT form) under `key`:
 *  1. d to coefficient form;
 *  2. for each digit j present at this level (primes j*alpha .. min((j+1)alpha, l)-1):
 *     its residues are kept on its own primes and base-converted to every other
 *     q_i (i < l) and to all special primes;
 *  3. the extended digit goes to NTT form;
 *  4. acc_b += ext_j * key_j.b, acc_a += ext_j * key_j.a on the l + K limbs;
 *  5. both accumulators are brought down by P (orc_mod_down).
 * Output ks0, ks1: l limbs each, NTT form, with ks0 + ks1*s ~ d*s'.
 */
/* steps 1-4 above: the two accumulators over the l + K limbs, before the division by P (zeroed here) */
void orc_key_switch_acc(const orc_ctx *c, const u64 *d, int l, const u64 *key, u64 *acc_b, u64 *acc_a) {
    u64 n = c->n;
    int total = c->L + c->K, ext = l + c->K;
    int digits = (l + c->alpha - 1) / c->alpha;
    u64 *dc = malloc((size_t)l * n * sizeof(u64));
    u64 *e = malloc(n * sizeof(u64));
    memset(acc_b, 0, (size_t)ext * n * sizeof(u64));
    memset(acc_a, 0, (size_t)ext * n * sizeof(u64));
    memcpy(dc, d, (size_t)l * n * sizeof(u64));
    for (int i = 0; i < l; i++) orc_intt(c, i, dc + (size_t)i * n);
    for (int j = 0; j < digits; j++) {
        int lo = j * c->alpha, hi = (j + 1) * c->alpha < l ? (j + 1) * c->alpha : l;
        const u64 *rows[ORC_MAX_PRIMES];
        int src[ORC_MAX_PRIMES];
        for (int i = lo; i < hi; i++) { rows[i - lo] = dc + (size_t)i * n; src[i - lo] = i; }
        for (int x = 0; x < ext; x++) {
            int prime = x < l ? x : c->L + (x - l); /* index into c->mod and into the key */
            if (prime >= lo && prime < hi) memcpy(e, dc + (size_t)prime * n, n * sizeof(u64));
            else orc_base_conv(c, rows, src, hi - lo, prime, e);
            orc_ntt(c, prime, e);
            u64 q = c->mod[prime];
            const u64 *kb = key + (((size_t)j * 2 + 0) * total + prime) * n;
            const u64 *ka = key + (((size_t)j * 2 + 1) * total + prime) * n;
            for (u64 t = 0; t < n; t++) {
                acc_b[(size_t)x * n + t] = addmod(acc_b[(size_t)x * n + t], mulmod(e[t], kb[t], q), q);
                acc_a[(size_t)x * n + t] = addmod(acc_a[(size_t)x * n + t], mulmod(e[t], ka[t], q), q);
            }
        }
    }
    free(dc); free(e);
}

void orc_key_switch(const orc_ctx *c, const u64 *d, int l, const u64 *key, u64 *ks0, u64 *ks1) {
    int ext = l + c->K;
    u64 *acc_b = malloc((size_t)ext * c->n * sizeof(u64));
    u64 *acc_a = malloc((size_t)ext * c->n * sizeof(u64));
    orc_key_switch_acc(c, d, l, key, acc_b, acc_a);
    orc_mod_down(c, acc_b, l, ks0);
    orc_mod_down(c, acc_a, l, ks1);
    free(acc_b); free(acc_a);
}

/*
 * Limb-wise multiply-accumulate on an arbitrary list of primes (indices into c->mod), for sums that are formed
 * before the division by P: acc[i] += x[i] * w[i] with one constant w[i] per limb (scalar) ...
 */
void orc_fma_const(const orc_ctx *c, u64 *acc, const u64 *x, const u64 *w_mod, const int *primes, int limbs) {
    u64 n = c->n;
    for (int i = 0; i < limbs; i++) {
        u64 q = c->mod[primes[i]];
        for (u64 j = 0; j < n; j++)
            acc[(size_t)i * n + j] = addmod(acc[(size_t)i * n + j], mulmod(x[(size_t)i * n + j], w_mod[i], q), q);
    }
}

/* ... or slot-wise with a plaintext given on the same primes, NTT form */
void orc_fma_plain(const orc_ctx *c, u64 *acc, const u64 *x, const u64 *pt, const int *primes, int limbs) {
    u64 n = c->n;
    for (int i = 0; i < limbs; i++) {
        u64 q = c->mod[primes[i]];
        for (u64 j = 0; j < n; j++)
            acc[(size_t)i * n + j] = addmod(acc[(size_t)i * n + j], mulmod(x[(size_t)i * n + j], pt[(size_t)i * n + j], q), q);
    }
}

/*
 * rotLeft: (sigma_g(c0) + ks0, ks1) with (ks0, ks1) the key switch of
 * sigma_g(c1) under the rotation key of g.  ct, out: [2][l][N].
 */
void orc_rotate(const orc_ctx *c, const u64 *ct, int l, u64 g, const u64 *key, u64 *out) {
    u64 n = c->n;
    u64 *r0 = malloc((size_t)l * n * sizeof(u64));
    u64 *r1 = malloc((size_t)l * n * sizeof(u64));
    orc_automorph_ntt(c, ct, g, 0, l, r0);
    orc_automorph_ntt(c, ct + (size_t)l * n, g, 0, l, r1);
    orc_key_switch(c, r1, l, key, out, out + (size_t)l * n);
    for (int i = 0; i < l; i++)
        for (u64 j = 0; j < n; j++)
            out[(size_t)i * n + j] = addmod(out[(size_t)i * n + j], r0[(size_t)i * n + j], c->mod[i]);
    free(r0); free(r1);
}

/* relinearize: (d0 + ks0, d1 + ks1) with (ks0, ks1) the key switch of d2 under the s^2 key */
void orc_relinearize(const orc_ctx *c, const u64 *ct3, int l, const u64 *key, u64 *out) {
    u64 n = c->n;
    orc_key_switch(c, ct3 + (size_t)2 * l * n, l, key, out, out + (size_t)l * n);
    for (int p = 0; p < 2; p++)
        for (int i = 0; i < l; i++)
            for (u64 j = 0; j < n; j++) {
                size_t o = ((size_t)p * l + i) * n + j;
                out[o] = addmod(out[o], ct3[o], c->mod[i]);
            }
}

/* ------------------------------------------------------------------ */
/* rescale = divScalar by the last modulus                             */
/* ------------------------------------------------------------------ */

/*
 * Per polynomial: the last limb goes to coefficient form; with h = floor(q_last/2)
 * the centred remainder of coefficient x is  r = ((x + h) mod q_last) - h, so that
 * (c - r)/q_last = floor((c + h)/q_last) coefficient-wise (round half up).  Then
 * for i < l-1:   out_i = (c_i - NTT_i(r mod q_i)) * q_last^-1 mod q_i.
 * ct [polys][l][N] -> out [polys][l-1][N].
 */
void orc_rescale(const orc_ctx *c, const u64 *ct, int polys, int l, u64 *out) {
    u64 n = c->n, ql = c->mod[l - 1], h = ql / 2;
    u64 *last = malloc(n * sizeof(u64));
    u64 *r = malloc(n * sizeof(u64));
    for (int p = 0; p < polys; p++) {
        memcpy(last, ct + ((size_t)p * l + (l - 1)) * n, n * sizeof(u64));
        orc_intt(c, l - 1, last);
        for (u64 j = 0; j < n; j++) last[j] = addmod(last[j], h, ql);
        for (int i = 0; i < l - 1; i++) {
            u64 q = c->mod[i];
            u64 ql_inv = invmod(ql % q, q);
            for (u64 j = 0; j < n; j++) r[j] = submod(last[j] % q, h % q, q);
            orc_ntt(c, i, r);
            for (u64 j = 0; j < n; j++) {
                u64 v = submod(ct[((size_t)p * l + i) * n + j], r[j], q);
                out[((size_t)p * (l - 1) + i) * n + j] = mulmod(v, ql_inv, q);
            }
        }
    }
    free(last); free(r);
}
