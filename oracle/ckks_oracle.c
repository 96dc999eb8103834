/*
 * CPU oracle for the RNS-CKKS ciphertext arithmetic (test infrastructure only).
 *
 * Plain, slow and meant to be checked by eye: every modular product is an
 * `unsigned __int128` product followed by `%`; the NTT is the textbook
 * iterative radix-2 loop; base conversion, ModDown and rescale are written as
 * the sums that define them.  No Montgomery, Barrett or Shoup arithmetic, no
 * blocking, no fusion.  It shares no code, header, table or constant with the
 * HIP library; only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.
 *
 * The paper (Section 2.2) names the CKKS operations Add, Mult, Rotate and
 * Bootstrap and defers every detail of the scheme to the CKKS literature; the
 * concrete algorithm steps below (full-RNS CKKS with hybrid key switching) are
 * the readings listed in the repository's design document.  Each function
 * names the step it implements.
 *
 * Layouts: a "limb" is N u64 residues in [0,q).  A ciphertext at level l (l =
 * number of limbs) is [2][l][N]; a switching key is [dnum][2][L+K][N] with
 * component 0 = b and 1 = a; moduli are indexed 0..L-1 (ciphertext primes
 * q_i) then L..L+K-1 (special primes p_k).  NTT-domain limbs are in
 * bit-reversed evaluation order.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

/* ---------------------------------------------------------------- scalars */

static u64 mulmod(u64 a, u64 b, u64 m) { return (u64)(((u128)a * b) % m); }
static u64 addmod(u64 a, u64 b, u64 m) { return (u64)(((u128)a + b) % m); }
static u64 submod(u64 a, u64 b, u64 m) { return (u64)(((u128)a + m - (b % m)) % m); }

static u64 powmod(u64 b, u64 e, u64 m)
{
    u64 r = 1 % m;
    b %= m;
    while (e) {
        if (e & 1) r = mulmod(r, b, m);
        b = mulmod(b, b, m);
        e >>= 1;
    }
    return r;
}

/* inverse modulo a prime (Fermat) */
static u64 invmod(u64 a, u64 m) { return powmod(a, m - 2, m); }

/* signed small integer -> residue in [0,m) */
static u64 lift_signed(i64 v, u64 m)
{
    if (v >= 0) return (u64)v % m;
    u64 a = (u64)(-(v + 1)) + 1; /* |v| without overflow */
    a %= m;
    return a ? m - a : 0;
}

static u64 bitrev(u64 x, int bits)
{
    u64 r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}

/* Least primitive root of the prime t: the smallest g whose order is t-1,
 * i.e. g^((t-1)/f) != 1 for every prime factor f of t-1 (trial division). */
u64 orc_least_primitive_root(u64 t)
{
    u64 fac[64];
    int nf = 0;
    u64 m = t - 1;
    for (u64 f = 2; f * f <= m; f += (f == 2 ? 1 : 2)) {
        if (m % f == 0) {
            fac[nf++] = f;
            while (m % f == 0) m /= f;
        }
    }
    if (m > 1) fac[nf++] = m;
    for (u64 g = 2; g < t; g++) {
        int ok = 1;
        for (int i = 0; i < nf && ok; i++)
            if (powmod(g, (t - 1) / fac[i], t) == 1) ok = 0;
        if (ok) return g;
    }
    return 0;
}

/* number of OpenMP threads the limb-parallel loops use (reported by the benchmark) */
int orc_num_threads(void) { return omp_get_max_threads(); }

/* ---------------------------------------------------------------- context */

typedef struct {
    int logN, L, K, dnum, alpha, M;
    u64 N;
    u64 *mod;     /* [M] */
    u64 *psi;     /* [M] primitive 2N-th root of unity */
    u64 *psi_br;  /* [M][N]  psi^{brv(i)}  */
    u64 *ipsi_br; /* [M][N]  psi^{-brv(i)} */
    u64 *ninv;    /* [M] N^{-1} */
    u64 cdt[38];  /* discrete-Gaussian cumulative thresholds, set by caller */
    int exact;    /* 0: fast (uncorrected) base conversions; 1: corrected ones (see orc_set_exact) */
} orc_ctx;

/* Context: moduli q_0..q_{L-1}, p_0..p_{K-1}; for each modulus t the root is
 * psi_t = g_t^((t-1)/2N) with g_t the least primitive root. */
orc_ctx *orc_ctx_create(int logN, int L, const u64 *q, int K, const u64 *p, int dnum)
{
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->logN = logN;
    c->N = (u64)1 << logN;
    c->L = L;
    c->K = K;
    c->dnum = dnum;
    c->alpha = (L + dnum - 1) / dnum;
    c->M = L + K;
    u64 N = c->N;
    c->mod = (u64 *)malloc(sizeof(u64) * c->M);
    c->psi = (u64 *)malloc(sizeof(u64) * c->M);
    c->ninv = (u64 *)malloc(sizeof(u64) * c->M);
    c->psi_br = (u64 *)malloc(sizeof(u64) * c->M * N);
    c->ipsi_br = (u64 *)malloc(sizeof(u64) * c->M * N);
    for (int i = 0; i < c->M; i++) c->mod[i] = i < L ? q[i] : p[i - L];
    for (int i = 0; i < c->M; i++) {
        u64 t = c->mod[i];
        if ((t - 1) % (2 * N) != 0) {
            /* caller error; leave tables zero */
            c->psi[i] = 0;
            continue;
        }
        u64 g = orc_least_primitive_root(t);
        u64 psi = powmod(g, (t - 1) / (2 * N), t);
        u64 ipsi = invmod(psi, t);
        c->psi[i] = psi;
        c->ninv[i] = invmod(N % t, t);
        /* psi^e for e = 0..N-1, stored at position brv(e) */
        u64 pw = 1, ipw = 1;
        for (u64 e = 0; e < N; e++) {
            u64 k = bitrev(e, logN);
            c->psi_br[(u64)i * N + k] = pw;
            c->ipsi_br[(u64)i * N + k] = ipw;
            pw = mulmod(pw, psi, t);
            ipw = mulmod(ipw, ipsi, t);
        }
    }
    return c;
}

void orc_ctx_destroy(orc_ctx *c)
{
    if (!c) return;
    free(c->mod);
    free(c->psi);
    free(c->ninv);
    free(c->psi_br);
    free(c->ipsi_br);
    free(c);
}

u64 orc_modulus(const orc_ctx *c, int i) { return c->mod[i]; }
u64 orc_psi(const orc_ctx *c, int i) { return c->psi[i]; }
int orc_alpha(const orc_ctx *c) { return c->alpha; }
void orc_set_cdt(orc_ctx *c, const u64 *cdt) { memcpy(c->cdt, cdt, sizeof(c->cdt)); }
/* Selects the corrected form of both base conversions (a separately specified variant, off by default).
 * The multiple v of the source modulus that the fast conversion leaves in its result is estimated in
 * double precision and taken out:
 *   ModUp:   v = floor(s),  s = sum over the digit's limbs, in order, of (double)y_i * (1.0 / (double)q_i);
 *            out_t = sum_i y_i [qhat_i]_t - v [D]_t  mod t, so the raised value is [x]_D in [0, D)
 *   ModDown: v = rint(s),   s = sum over k, in order, of (double)y'_k * (1.0 / (double)p_k), y'_k the centred digit;
 *            r_i = sum_k y'_k [Phat_k]_{q_i} - v [P]_{q_i}  mod q_i, so r is the centred [u]_P and the result
 *            (u - r)/P is u/P rounded to nearest
 * Every product and sum of s is one IEEE double operation (no fused multiply-add), rint rounds halves to even.
 * When the exact sum lies within the rounding error of s (about 2^-50) of an integer (ModUp) or of a half
 * (ModDown), v can be one off and the result is the exact one plus or minus one source modulus: still a valid
 * conversion, and the same on every implementation that follows this definition. */
void orc_set_exact(orc_ctx *c, int exact) { c->exact = exact; }

/* index of the modulus held by active limb a at level lvl:
 * a < lvl -> q_a, otherwise special prime p_{a-lvl}. */
static int active_mod(const orc_ctx *c, int lvl, int a) { return a < lvl ? a : c->L + (a - lvl); }

/* ------------------------------------------------------------------- NTT */

/* Forward negacyclic NTT of one limb, in place:
 *   out[k] = sum_j a[j] * psi^((2*brv(k)+1)*j)  mod q.
 * Textbook decimation-in-time loop with the powers of psi stored in
 * bit-reversed order; it emits the evaluations in bit-reversed order. */
void orc_ntt(const orc_ctx *c, int mi, u64 *a)
{
    u64 N = c->N, q = c->mod[mi];
    const u64 *w = c->psi_br + (u64)mi * N;
    u64 t = N;
    for (u64 m = 1; m < N; m *= 2) {
        t /= 2;
        for (u64 i = 0; i < m; i++) {
            u64 S = w[m + i];
            u64 j1 = 2 * i * t;
            for (u64 j = j1; j < j1 + t; j++) {
                u64 U = a[j];
                u64 V = mulmod(a[j + t], S, q);
                a[j] = addmod(U, V, q);
                a[j + t] = submod(U, V, q);
            }
        }
    }
}

/* Inverse of orc_ntt (decimation in frequency, then the factor 1/N). */
void orc_intt(const orc_ctx *c, int mi, u64 *a)
{
    u64 N = c->N, q = c->mod[mi];
    const u64 *w = c->ipsi_br + (u64)mi * N;
    u64 t = 1;
    for (u64 m = N; m > 1; m /= 2) {
        u64 h = m / 2;
        u64 j1 = 0;
        for (u64 i = 0; i < h; i++) {
            u64 S = w[h + i];
            for (u64 j = j1; j < j1 + t; j++) {
                u64 U = a[j];
                u64 V = a[j + t];
                a[j] = addmod(U, V, q);
                a[j + t] = mulmod(submod(U, V, q), S, q);
            }
            j1 += 2 * t;
        }
        t *= 2;
    }
    for (u64 j = 0; j < N; j++) a[j] = mulmod(a[j], c->ninv[mi], q);
}

/* One output of the forward NTT straight from its definition (O(N)):
 * the polynomial a evaluated at psi^(2*brv(k)+1). */
u64 orc_ntt_direct_at(const orc_ctx *c, int mi, const u64 *a, u64 k)
{
    u64 N = c->N, q = c->mod[mi];
    u64 e = 2 * bitrev(k, c->logN) + 1;
    u64 x = powmod(c->psi[mi], e, q);
    u64 acc = 0, xp = 1;
    for (u64 j = 0; j < N; j++) {
        acc = addmod(acc, mulmod(a[j] % q, xp, q), q);
        xp = mulmod(xp, x, q);
    }
    return acc;
}

/* batch helpers: limbs [B][N], modulus index per limb */
void orc_ntt_batch(const orc_ctx *c, u64 *a, const int *mi, int B)
{
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; b++) orc_ntt(c, mi[b], a + (u64)b * c->N);
}

void orc_intt_batch(const orc_ctx *c, u64 *a, const int *mi, int B)
{
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; b++) orc_intt(c, mi[b], a + (u64)b * c->N);
}

/* ------------------------------------------------------------ randomness */

/* Counter-based generator: word i of the stream (seed, tag) is
 * mix(key + (i+1)*GAMMA), key = mix(mix(seed + GAMMA) + tag*GAMMA), with the
 * SplitMix64 finaliser as mix. */
#define ORC_GAMMA 0x9E3779B97F4A7C15ull
static u64 mix64(u64 z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static u64 stream_key(u64 seed, u64 tag) { return mix64(mix64(seed + ORC_GAMMA) + tag * ORC_GAMMA); }
u64 orc_stream_word(u64 seed, u64 tag, u64 i) { return mix64(stream_key(seed, tag) + (i + 1) * ORC_GAMMA); }

/* tag = kind<<32 | a<<16 | b.  kinds: 1 secret, 2 key mask a_j, 3 key error
 * e_j, 4 encryption mask, 5 encryption error. */
static u64 mktag(u64 kind, u64 a, u64 b) { return (kind << 32) | (a << 16) | b; }

/* uniform in [0,q): keep the low bitlen(q) bits of each word, reject >= q */
void orc_sample_uniform(u64 seed, u64 tag, u64 q, u64 *out, u64 n)
{
    int bits = 0;
    while (bits < 64 && (q >> bits)) bits++;
    u64 mask = bits == 64 ? ~(u64)0 : (((u64)1 << bits) - 1);
    u64 key = stream_key(seed, tag), ctr = 0;
    for (u64 k = 0; k < n; k++) {
        u64 v;
        do {
            ctr++;
            v = mix64(key + ctr * ORC_GAMMA) & mask;
        } while (v >= q);
        out[k] = v;
    }
}

/* ternary: reject words >= 3*floor(2^64/3); word mod 3 = 0,1,2 -> 0,+1,-1 */
void orc_sample_ternary(u64 seed, u64 tag, int8_t *out, u64 n)
{
    const u64 lim = 3 * (0xFFFFFFFFFFFFFFFFull / 3);
    u64 key = stream_key(seed, tag), ctr = 0;
    for (u64 k = 0; k < n; k++) {
        u64 v;
        do {
            ctr++;
            v = mix64(key + ctr * ORC_GAMMA);
        } while (v >= lim);
        u64 r = v % 3;
        out[k] = r == 0 ? 0 : (r == 1 ? 1 : -1);
    }
}

/* discrete Gaussian on [-19,19]: one word per sample, value = -19 + number
 * of cumulative thresholds that the word reaches. */
void orc_sample_gauss(const orc_ctx *c, u64 seed, u64 tag, int8_t *out, u64 n)
{
    u64 key = stream_key(seed, tag);
    for (u64 k = 0; k < n; k++) {
        u64 u = mix64(key + (k + 1) * ORC_GAMMA);
        int v = -19;
        for (int t = 0; t < 38; t++)
            if (u >= c->cdt[t]) v++;
        out[k] = (int8_t)v;
    }
}

/* ------------------------------------------------------ encode / decode */

/* Slot j sits at zeta_j = zeta^(5^j mod 2N), zeta = exp(i*pi/N).
 * Encode: m_k = rint(scale * (2/N) * Re sum_j z_j * zeta_j^(-k)). */
void orc_encode(const orc_ctx *c, const double *re, const double *im, double scale, i64 *out)
{
    u64 N = c->N, n = N / 2, twoN = 2 * N;
    double *cs = (double *)malloc(sizeof(double) * twoN);
    double *sn = (double *)malloc(sizeof(double) * twoN);
    u64 *pw = (u64 *)malloc(sizeof(u64) * n);
    for (u64 e = 0; e < twoN; e++) {
        cs[e] = cos(M_PI * (double)e / (double)N);
        sn[e] = sin(M_PI * (double)e / (double)N);
    }
    u64 g = 1;
    for (u64 j = 0; j < n; j++) {
        pw[j] = g;
        g = (g * 5) % twoN;
    }
#pragma omp parallel for schedule(static)
    for (u64 k = 0; k < N; k++) {
        double acc = 0.0;
        for (u64 j = 0; j < n; j++) {
            u64 e = (pw[j] * k) % twoN;
            /* Re( z * conj(zeta^e) ) */
            double zi = im ? im[j] : 0.0;
            acc += re[j] * cs[e] + zi * sn[e];
        }
        out[k] = (i64)rint(scale * (2.0 / (double)N) * acc);
    }
    free(cs);
    free(sn);
    free(pw);
}

/* Decode: z_j = (1/scale) * sum_k m_k * zeta_j^k, m given as doubles. */
void orc_decode(const orc_ctx *c, const double *m, double scale, double *re, double *im)
{
    u64 N = c->N, n = N / 2, twoN = 2 * N;
    double *cs = (double *)malloc(sizeof(double) * twoN);
    double *sn = (double *)malloc(sizeof(double) * twoN);
    for (u64 e = 0; e < twoN; e++) {
        cs[e] = cos(M_PI * (double)e / (double)N);
        sn[e] = sin(M_PI * (double)e / (double)N);
    }
    u64 *pw = (u64 *)malloc(sizeof(u64) * n);
    u64 g = 1;
    for (u64 j = 0; j < n; j++) {
        pw[j] = g;
        g = (g * 5) % twoN;
    }
#pragma omp parallel for schedule(static)
    for (u64 j = 0; j < n; j++) {
        double ar = 0.0, ai = 0.0;
        for (u64 k = 0; k < N; k++) {
            u64 e = (pw[j] * k) % twoN;
            ar += m[k] * cs[e];
            ai += m[k] * sn[e];
        }
        re[j] = ar / scale;
        im[j] = ai / scale;
    }
    free(cs);
    free(sn);
    free(pw);
}

/* --------------------------------------------------------- automorphism */

/* sigma_g in the coefficient domain: a(X) -> a(X^g) in Z_t[X]/(X^N+1).
 * Coefficient j moves to j*g mod 2N; an index >= N wraps with a sign flip. */
void orc_automorph_coeff(const orc_ctx *c, int mi, u64 g, const u64 *in, u64 *out)
{
    u64 N = c->N, t = c->mod[mi];
    for (u64 j = 0; j < N; j++) {
        u64 e = (u64)(((u128)j * g) % (2 * N));
        if (e < N)
            out[e] = in[j];
        else
            out[e - N] = in[j] ? t - in[j] : 0;
    }
}

/* same on a small signed polynomial (the secret) */
void orc_automorph_small(const orc_ctx *c, u64 g, const int8_t *in, int8_t *out)
{
    u64 N = c->N;
    for (u64 j = 0; j < N; j++) {
        u64 e = (u64)(((u128)j * g) % (2 * N));
        if (e < N)
            out[e] = in[j];
        else
            out[e - N] = (int8_t)(-in[j]);
    }
}

/* Galois element of a left rotation by r slots: 5^r mod 2N (r may be
 * negative: the inverse power). */
u64 orc_galois_element(const orc_ctx *c, i64 r)
{
    u64 twoN = 2 * c->N, n = c->N / 2;
    i64 rr = r % (i64)n;
    if (rr < 0) rr += (i64)n;
    u64 g = 1;
    for (i64 i = 0; i < rr; i++) g = (g * 5) % twoN;
    return g;
}

/* ------------------------------------------------------ keys and encrypt */

/* secret: ternary coefficients */
void orc_keygen_secret(const orc_ctx *c, u64 seed, int8_t *s)
{
    orc_sample_ternary(seed, mktag(1, 0, 0), s, c->N);
}

/* small signed polynomial -> NTT form for modulus mi */
void orc_small_to_ntt(const orc_ctx *c, int mi, const int8_t *s, u64 *out)
{
    for (u64 j = 0; j < c->N; j++) out[j] = lift_signed(s[j], c->mod[mi]);
    orc_ntt(c, mi, out);
}

/* Switching key from s' to s (hybrid key switching with dnum digits):
 * for each digit j and modulus i: a_j[i] uniform, e_j Gaussian,
 *   b_j[i] = -a_j[i]*s[i] + NTT_i(e_j) + (q_i in digit j ? [P]_{q_i} * s'[i] : 0)
 * with P the product of the special primes.  sp_ntt holds s' in NTT form for
 * the L ciphertext moduli.  evk layout [dnum][2][M][N]. */
void orc_keygen_switch(const orc_ctx *c, const int8_t *s, const u64 *sp_ntt, u64 seed, u64 *evk)
{
    u64 N = c->N;
    int M = c->M;
    int8_t *e = (int8_t *)malloc(N);
    for (int j = 0; j < c->dnum; j++) {
        orc_sample_gauss(c, seed, mktag(3, (u64)j, 0), e, N);
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < M; i++) {
            u64 t = c->mod[i];
            u64 *b = evk + (((u64)j * 2 + 0) * M + i) * N;
            u64 *a = evk + (((u64)j * 2 + 1) * M + i) * N;
            u64 *sh = (u64 *)malloc(sizeof(u64) * N);
            u64 *eh = (u64 *)malloc(sizeof(u64) * N);
            orc_sample_uniform(seed, mktag(2, (u64)j, (u64)i), t, a, N);
            orc_small_to_ntt(c, i, s, sh);
            orc_small_to_ntt(c, i, e, eh);
            u64 Pmod = 1;
            int in_digit = (i < c->L) && (i / c->alpha == j);
            if (in_digit)
                for (int k = 0; k < c->K; k++) Pmod = mulmod(Pmod, c->mod[c->L + k] % t, t);
            for (u64 x = 0; x < N; x++) {
                u64 v = submod(eh[x], mulmod(a[x], sh[x], t), t);
                if (in_digit) v = addmod(v, mulmod(Pmod, sp_ntt[(u64)i * N + x], t), t);
                b[x] = v;
            }
            free(sh);
            free(eh);
        }
    }
    free(e);
}

/* Symmetric encryption of the integer polynomial m at level lvl:
 * c1[i] = a_i uniform (taken as NTT-domain values),
 * c0[i] = -a_i*s_i + NTT_i(e) + NTT_i(m). */
void orc_encrypt(const orc_ctx *c, const int8_t *s, const i64 *m, int lvl, u64 seed, u64 *ct)
{
    u64 N = c->N;
    int8_t *e = (int8_t *)malloc(N);
    orc_sample_gauss(c, seed, mktag(5, 0, 0), e, N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < lvl; i++) {
        u64 t = c->mod[i];
        u64 *c0 = ct + ((u64)0 * lvl + i) * N;
        u64 *c1 = ct + ((u64)1 * lvl + i) * N;
        u64 *sh = (u64 *)malloc(sizeof(u64) * N);
        u64 *eh = (u64 *)malloc(sizeof(u64) * N);
        u64 *mh = (u64 *)malloc(sizeof(u64) * N);
        orc_sample_uniform(seed, mktag(4, 0, (u64)i), t, c1, N);
        orc_small_to_ntt(c, i, s, sh);
        orc_small_to_ntt(c, i, e, eh);
        for (u64 x = 0; x < N; x++) mh[x] = lift_signed(m[x], t);
        orc_ntt(c, i, mh);
        for (u64 x = 0; x < N; x++) {
            u64 v = submod(eh[x], mulmod(c1[x], sh[x], t), t);
            c0[x] = addmod(v, mh[x], t);
        }
        free(sh);
        free(eh);
        free(mh);
    }
    free(e);
}

/* Decryption up to the CRT step: out[i] = iNTT_i(c0[i] + c1[i]*s_i), i<lvl.
 * The caller reconstructs the centred integer from the residues. */
void orc_decrypt_residues(const orc_ctx *c, const int8_t *s, const u64 *ct, int lvl, u64 *out)
{
    u64 N = c->N;
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < lvl; i++) {
        u64 t = c->mod[i];
        const u64 *c0 = ct + ((u64)0 * lvl + i) * N;
        const u64 *c1 = ct + ((u64)1 * lvl + i) * N;
        u64 *o = out + (u64)i * N;
        u64 *sh = (u64 *)malloc(sizeof(u64) * N);
        orc_small_to_ntt(c, i, s, sh);
        for (u64 x = 0; x < N; x++) o[x] = addmod(c0[x], mulmod(c1[x], sh[x], t), t);
        orc_intt(c, i, o);
        free(sh);
    }
}

/* ---------------------------------------------------------- elementwise */

/* op: 0 add, 1 sub, 2 mul; limbs [B][N], limb b uses modulus index mi[b] */
void orc_limbwise(const orc_ctx *c, int op, const u64 *a, const u64 *b, u64 *out, const int *mi, int B)
{
    u64 N = c->N;
#pragma omp parallel for schedule(static)
    for (int l = 0; l < B; l++) {
        u64 t = c->mod[mi[l]];
        for (u64 x = 0; x < N; x++) {
            u64 u = a[(u64)l * N + x], v = b[(u64)l * N + x], r;
            if (op == 0)
                r = addmod(u, v, t);
            else if (op == 1)
                r = submod(u, v, t);
            else
                r = mulmod(u, v, t);
            out[(u64)l * N + x] = r;
        }
    }
}

/* ct * plaintext (NTT-domain plaintext [lvl][N]) */
void orc_pmult(const orc_ctx *c, const u64 *ct, const u64 *pt, int lvl, u64 *out)
{
    u64 N = c->N;
    for (int comp = 0; comp < 2; comp++)
#pragma omp parallel for schedule(static)
        for (int i = 0; i < lvl; i++) {
            u64 t = c->mod[i];
            const u64 *a = ct + ((u64)comp * lvl + i) * N;
            const u64 *p = pt + (u64)i * N;
            u64 *o = out + ((u64)comp * lvl + i) * N;
            for (u64 x = 0; x < N; x++) o[x] = mulmod(a[x], p[x], t);
        }
}

/* ct * per-limb scalar (scalar[i] in [0,q_i)) */
void orc_cmult(const orc_ctx *c, const u64 *ct, const u64 *scalar, int lvl, u64 *out)
{
    u64 N = c->N;
    for (int comp = 0; comp < 2; comp++)
        for (int i = 0; i < lvl; i++) {
            u64 t = c->mod[i];
            const u64 *a = ct + ((u64)comp * lvl + i) * N;
            u64 *o = out + ((u64)comp * lvl + i) * N;
            for (u64 x = 0; x < N; x++) o[x] = mulmod(a[x], scalar[i] % t, t);
        }
}

/* ct + constant: a constant polynomial c has the value c at every evaluation point, so adding the
 * plaintext constant scalar[i] (a residue of q_i) adds it to every NTT coefficient of c0. */
void orc_add_const(const orc_ctx *c, const u64 *ct, const u64 *scalar, int lvl, u64 *out)
{
    u64 N = c->N;
    memcpy(out, ct, sizeof(u64) * 2 * lvl * N);
    for (int i = 0; i < lvl; i++) {
        u64 t = c->mod[i];
        for (u64 x = 0; x < N; x++) out[(u64)i * N + x] = addmod(ct[(u64)i * N + x], scalar[i] % t, t);
    }
}

/* Tensor product of two level-lvl ciphertexts, NTT domain:
 * d0 = a0*b0, d1 = a0*b1 + a1*b0, d2 = a1*b1.  out [3][lvl][N]. */
void orc_tensor(const orc_ctx *c, const u64 *A, const u64 *B, int lvl, u64 *out)
{
    u64 N = c->N;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < lvl; i++) {
        u64 t = c->mod[i];
        const u64 *a0 = A + (u64)i * N, *a1 = A + ((u64)lvl + i) * N;
        const u64 *b0 = B + (u64)i * N, *b1 = B + ((u64)lvl + i) * N;
        u64 *d0 = out + (u64)i * N, *d1 = out + ((u64)lvl + i) * N, *d2 = out + ((u64)2 * lvl + i) * N;
        for (u64 x = 0; x < N; x++) {
            d0[x] = mulmod(a0[x], b0[x], t);
            d1[x] = addmod(mulmod(a0[x], b1[x], t), mulmod(a1[x], b0[x], t), t);
            d2[x] = mulmod(a1[x], b1[x], t);
        }
    }
}

/* --------------------------------------------------------- key switching */

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* Digit decomposition + ModUp (fast basis conversion, no correction of the
 * overshoot).  x: coefficient-domain limbs [lvl][N].  For each active digit j
 * with active limb set C, D = prod_{i in C} q_i, qhat_i = D/q_i:
 *   y_i = x_i * [qhat_i^{-1}]_{q_i} mod q_i               (value in [0,q_i))
 *   out[j][a] = sum_{i in C} y_i * [qhat_i]_t  mod t      for t outside C
 *   out[j][a] = x_a                                        for t inside C
 * out: coefficient domain, [beta][lvl+K][N]. */
void orc_modup(const orc_ctx *c, const u64 *x, int lvl, u64 *out)
{
    u64 N = c->N;
    int Ma = lvl + c->K, beta = ceil_div(lvl, c->alpha);
    for (int j = 0; j < beta; j++) {
        int lo = j * c->alpha, hi = (j + 1) * c->alpha;
        if (hi > lvl) hi = lvl;
        int na = hi - lo;
        u64 *y = (u64 *)malloc(sizeof(u64) * na * N);
        for (int ii = 0; ii < na; ii++) {
            u64 qi = c->mod[lo + ii];
            u64 qhat = 1;
            for (int i2 = lo; i2 < hi; i2++)
                if (i2 != lo + ii) qhat = mulmod(qhat, c->mod[i2] % qi, qi);
            u64 inv = invmod(qhat, qi);
            for (u64 n = 0; n < N; n++) y[(u64)ii * N + n] = mulmod(x[(u64)(lo + ii) * N + n], inv, qi);
        }
#pragma omp parallel for schedule(dynamic)
        for (int a = 0; a < Ma; a++) {
            int mi = active_mod(c, lvl, a);
            u64 t = c->mod[mi];
            u64 *o = out + ((u64)j * Ma + a) * N;
            if (a >= lo && a < hi) {
                memcpy(o, x + (u64)a * N, sizeof(u64) * N);
                continue;
            }
            for (u64 n = 0; n < N; n++) o[n] = 0;
            for (int ii = 0; ii < na; ii++) {
                u64 qhat_t = 1;
                for (int i2 = lo; i2 < hi; i2++)
                    if (i2 != lo + ii) qhat_t = mulmod(qhat_t, c->mod[i2] % t, t);
                for (u64 n = 0; n < N; n++)
                    o[n] = addmod(o[n], mulmod(y[(u64)ii * N + n] % t, qhat_t, t), t);
            }
            if (c->exact) { /* take out v D, v = floor(sum_i y_i / q_i) in double precision */
                u64 D_t = 1;
                for (int i2 = lo; i2 < hi; i2++) D_t = mulmod(D_t, c->mod[i2] % t, t);
                for (u64 n = 0; n < N; n++) {
                    double sum = 0.0; /* built with -ffp-contract=off: one IEEE rounding per operation */
                    for (int ii = 0; ii < na; ii++) {
                        double rq = 1.0 / (double)c->mod[lo + ii];
                        sum = sum + (double)y[(u64)ii * N + n] * rq;
                    }
                    u64 v = (u64)floor(sum);
                    o[n] = submod(o[n], mulmod(v, D_t, t), t);
                }
            }
        }
        free(y);
    }
}

/* ModDown of one polynomial u given in the NTT domain on lvl+K limbs, with centred conversion
 * digits:
 *   w_k = iNTT(u[p_k]);  y_k = w_k * [Phat_k^{-1}]_{p_k} mod p_k, then centred:
 *         y_k - p_k if y_k > (p_k-1)/2
 *   r_i = sum_k y_k * [Phat_k]_{q_i} mod q_i               (per coefficient, uncorrected)
 *   out[i] = (u[i] - NTT_i(r_i)) * [P^{-1}]_{q_i} mod q_i.
 * As integers r = [u]_P + v P with r in (-K P/2, K P/2), so out = (u - r)/P = u/P - r/P: the
 * error r/P is symmetric about zero (no systematic bias), |r/P| < K/2.
 * out: NTT domain, [lvl][N]. */
void orc_moddown(const orc_ctx *c, const u64 *u, int lvl, u64 *out)
{
    u64 N = c->N;
    int K = c->K, L = c->L;
    u64 *y = (u64 *)malloc(sizeof(u64) * K * N);
    for (int k = 0; k < K; k++) {
        u64 pk = c->mod[L + k];
        u64 *w = y + (u64)k * N;
        memcpy(w, u + (u64)(lvl + k) * N, sizeof(u64) * N);
        orc_intt(c, L + k, w);
        u64 phat = 1;
        for (int k2 = 0; k2 < K; k2++)
            if (k2 != k) phat = mulmod(phat, c->mod[L + k2] % pk, pk);
        u64 inv = invmod(phat, pk);
        for (u64 n = 0; n < N; n++) w[n] = mulmod(w[n], inv, pk);
    }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < lvl; i++) {
        u64 qi = c->mod[i];
        u64 *r = (u64 *)calloc(N, sizeof(u64));
        u64 Pmod = 1;
        for (int k = 0; k < K; k++) Pmod = mulmod(Pmod, c->mod[L + k] % qi, qi);
        u64 Pinv = invmod(Pmod, qi);
        for (int k = 0; k < K; k++) {
            u64 pk = c->mod[L + k];
            u64 phat_q = 1;
            for (int k2 = 0; k2 < K; k2++)
                if (k2 != k) phat_q = mulmod(phat_q, c->mod[L + k2] % qi, qi);
            for (u64 n = 0; n < N; n++) {
                u64 yk = y[(u64)k * N + n];
                u64 term;
                if (yk > (pk - 1) / 2) /* negative digit y_k - p_k */
                    term = submod(0, mulmod((pk - yk) % qi, phat_q, qi), qi);
                else
                    term = mulmod(yk % qi, phat_q, qi);
                r[n] = addmod(r[n], term, qi);
            }
        }
        if (c->exact) { /* take out v P, v = rint(sum_k y'_k / p_k) in double precision, y' the centred digits */
            for (u64 n = 0; n < N; n++) {
                double sum = 0.0;
                for (int k = 0; k < K; k++) {
                    u64 pk = c->mod[L + k], yk = y[(u64)k * N + n];
                    double rp = 1.0 / (double)pk;
                    double yc = yk > (pk - 1) / 2 ? -(double)(pk - yk) : (double)yk;
                    sum = sum + yc * rp;
                }
                double v = rint(sum);
                if (v >= 0.0)
                    r[n] = submod(r[n], mulmod((u64)v, Pmod, qi), qi);
                else
                    r[n] = addmod(r[n], mulmod((u64)(-v), Pmod, qi), qi);
            }
        }
        orc_ntt(c, i, r);
        for (u64 n = 0; n < N; n++) out[(u64)i * N + n] = mulmod(submod(u[(u64)i * N + n], r[n], qi), Pinv, qi);
        free(r);
    }
    free(y);
}

/* KeySwitch(d, evk) at level lvl; d in the NTT domain [lvl][N]; g = Galois
 * element applied to the raised digits (1 = none).  Steps: iNTT, ModUp,
 * (sigma_g in the coefficient domain), NTT, inner product with the key over
 * the lvl+K active moduli, ModDown of both components.
 * raised_out (nullable): NTT-domain raised digits [beta][lvl+K][N].
 * u_out (nullable): inner products [2][lvl+K][N]. */
void orc_keyswitch(const orc_ctx *c, const u64 *d, int lvl, const u64 *evk, u64 g, u64 *k0, u64 *k1,
                   u64 *raised_out, u64 *u_out)
{
    u64 N = c->N;
    int Ma = lvl + c->K, M = c->M, beta = ceil_div(lvl, c->alpha);
    u64 *x = (u64 *)malloc(sizeof(u64) * lvl * N);
    memcpy(x, d, sizeof(u64) * lvl * N);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < lvl; i++) orc_intt(c, i, x + (u64)i * N);
    u64 *raised = (u64 *)malloc(sizeof(u64) * beta * Ma * N);
    orc_modup(c, x, lvl, raised);
#pragma omp parallel for schedule(dynamic)
    for (int ja = 0; ja < beta * Ma; ja++) {
        int a = ja % Ma;
        int mi = active_mod(c, lvl, a);
        u64 *limb = raised + (u64)ja * N;
        if (g != 1) {
            u64 *tmp = (u64 *)malloc(sizeof(u64) * N);
            orc_automorph_coeff(c, mi, g, limb, tmp);
            memcpy(limb, tmp, sizeof(u64) * N);
            free(tmp);
        }
        orc_ntt(c, mi, limb);
    }
    if (raised_out) memcpy(raised_out, raised, sizeof(u64) * beta * Ma * N);
    u64 *u = (u64 *)calloc((u64)2 * Ma * N, sizeof(u64));
#pragma omp parallel for schedule(dynamic)
    for (int ca = 0; ca < 2 * Ma; ca++) {
        int comp = ca / Ma, a = ca % Ma;
        int mi = active_mod(c, lvl, a);
        u64 t = c->mod[mi];
        u64 *o = u + (u64)ca * N;
        for (int j = 0; j < beta; j++) {
            const u64 *dj = raised + ((u64)j * Ma + a) * N;
            const u64 *kj = evk + (((u64)j * 2 + comp) * M + mi) * N;
            for (u64 n = 0; n < N; n++) o[n] = addmod(o[n], mulmod(dj[n], kj[n], t), t);
        }
    }
    if (u_out) memcpy(u_out, u, sizeof(u64) * 2 * Ma * N);
    orc_moddown(c, u, lvl, k0);
    orc_moddown(c, u + (u64)Ma * N, lvl, k1);
    free(x);
    free(raised);
    free(u);
}

/* HMult with relinearisation (no rescale): (d0,d1,d2) = tensor product;
 * (k0,k1) = KeySwitch(d2, relin key); out = (d0+k0, d1+k1). */
void orc_hmult_relin(const orc_ctx *c, const u64 *A, const u64 *B, int lvl, const u64 *evk, u64 *out)
{
    u64 N = c->N;
    u64 *d = (u64 *)malloc(sizeof(u64) * 3 * lvl * N);
    u64 *k = (u64 *)malloc(sizeof(u64) * 2 * lvl * N);
    orc_tensor(c, A, B, lvl, d);
    orc_keyswitch(c, d + (u64)2 * lvl * N, lvl, evk, 1, k, k + (u64)lvl * N, NULL, NULL);
    for (int comp = 0; comp < 2; comp++)
        for (int i = 0; i < lvl; i++) {
            u64 t = c->mod[i];
            u64 off = ((u64)comp * lvl + i) * N;
            for (u64 n = 0; n < N; n++) out[off + n] = addmod(d[off + n], k[off + n], t);
        }
    free(d);
    free(k);
}

/* Rescale: drop the last limb q_last with centred rounding.  Per component:
 * r = iNTT(c[lvl-1]) in [0,q_last); r_c = r - q_last if r > (q_last-1)/2;
 * out[i] = (c[i] - NTT_i(r_c mod q_i)) * [q_last^{-1}]_{q_i} mod q_i, i<lvl-1.
 * out [2][lvl-1][N]. */
void orc_rescale(const orc_ctx *c, const u64 *ct, int lvl, u64 *out)
{
    u64 N = c->N;
    int last = lvl - 1;
    u64 ql = c->mod[last];
    for (int comp = 0; comp < 2; comp++) {
        u64 *r = (u64 *)malloc(sizeof(u64) * N);
        memcpy(r, ct + ((u64)comp * lvl + last) * N, sizeof(u64) * N);
        orc_intt(c, last, r);
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < last; i++) {
            u64 qi = c->mod[i];
            u64 *ri = (u64 *)malloc(sizeof(u64) * N);
            for (u64 n = 0; n < N; n++) {
                if (r[n] > (ql - 1) / 2) {
                    /* negative representative r - q_last */
                    u64 mag = (ql - r[n]) % qi;
                    ri[n] = mag ? qi - mag : 0;
                } else
                    ri[n] = r[n] % qi;
            }
            orc_ntt(c, i, ri);
            u64 qlinv = invmod(ql % qi, qi);
            const u64 *src = ct + ((u64)comp * lvl + i) * N;
            u64 *dst = out + ((u64)comp * last + i) * N;
            for (u64 n = 0; n < N; n++) dst[n] = mulmod(submod(src[n], ri[n], qi), qlinv, qi);
            free(ri);
        }
        free(r);
    }
}

/* HRot by the Galois element g (g = 5^r for a left rotation by r slots):
 * key switch of c1 with the automorphism applied to the raised digits, and
 * out = (sigma_g(c0) + k0, k1).  sigma_g(c0) is taken by its definition:
 * iNTT, coefficient permutation with signs, NTT. */
void orc_hrot(const orc_ctx *c, const u64 *ct, int lvl, const u64 *evk, u64 g, u64 *out)
{
    u64 N = c->N;
    orc_keyswitch(c, ct + (u64)lvl * N, lvl, evk, g, out, out + (u64)lvl * N, NULL, NULL);
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < lvl; i++) {
        u64 t = c->mod[i];
        u64 *a = (u64 *)malloc(sizeof(u64) * N);
        u64 *b = (u64 *)malloc(sizeof(u64) * N);
        memcpy(a, ct + (u64)i * N, sizeof(u64) * N);
        orc_intt(c, i, a);
        orc_automorph_coeff(c, i, g, a, b);
        orc_ntt(c, i, b);
        for (u64 n = 0; n < N; n++) out[(u64)i * N + n] = addmod(out[(u64)i * N + n], b[n], t);
        free(a);
        free(b);
    }
}
