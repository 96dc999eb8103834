/*
 * he.h -- C ABI of the MI355X RNS-CKKS ciphertext-arithmetic library.
 *
 * The paper (Section 2.2) builds its encrypted logistic regression from the CKKS
 * operations Add, Mult (slot-wise product, one level consumed) and Rotate and
 * defers the scheme itself to the CKKS literature.  This library implements the
 * full-RNS form of those operations with hybrid key switching (dnum digits,
 * K special primes): negacyclic NTT/iNTT, tensor product + relinearisation,
 * slot rotation (ModUp, inner product with the evaluation key, ModDown),
 * rescale, and rotate-and-sum.  Key generation, encoding, encryption and
 * decryption run on the host; everything else runs in HIP kernels (gfx950) on
 * device buffers owned by the caller.
 *
 * Conventions
 *  - Moduli: q_0..q_{L-1} (ciphertext primes) then p_0..p_{K-1} (special primes),
 *    all < 2^60, all = 1 mod 2N.  "Modulus index" i < L means q_i, L+k means p_k.
 *  - level l = number of limbs present (1..L).  A limb is N uint64 residues in
 *    [0, q).  Every buffer that crosses this interface holds canonical residues.
 *  - NTT domain: out[k] = sum_j a[j] psi^((2 brv(k)+1) j) mod q (bit-reversed
 *    evaluation order), psi = g^((q-1)/2N) with g the least primitive root of q.
 *  - Ciphertext: uint64 [2][l][N], NTT domain, component 0 = c0, 1 = c1;
 *    decryption is c0 + c1*s.  Evaluation key: uint64 [dnum][2][L+K][N],
 *    component 0 = b, 1 = a.
 *  - Slots: n = N/2 complex values; slot j is the evaluation at
 *    exp(i pi 5^j / N).  Rotation by r is the left cyclic shift
 *    out[j] = in[(j+r) mod n].
 *  - Scale and level are tracked by the caller; the library checks levels only.
 *  - "h_" arguments are host pointers, "d_" arguments are device pointers
 *    (hipMalloc'ed or a torch tensor's data_ptr), contiguous and 16-byte aligned,
 *    owned by the caller.  `stream` is a hipStream_t passed as void* (NULL = the
 *    default stream).  Device functions only enqueue work: they never
 *    synchronise and never allocate; results are valid once the stream reaches
 *    the end of the enqueued work.  Output buffers may alias an input only
 *    where stated.
 *  - Every function returns HE_OK (0) or a negative error code; nothing throws
 *    or aborts.  Handles are freed with the matching _destroy.
 */
#ifndef HE_H_
#define HE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HE_OK 0
#define HE_EINVAL (-1)     /* null pointer, bad size, modulus not = 1 mod 2N, ... */
#define HE_ELEVEL (-2)     /* level out of range, or level 1 cannot be rescaled */
#define HE_ENOKEY (-3)     /* key handle missing or of the wrong kind */
#define HE_EWORKSPACE (-4) /* workspace too small */
#define HE_EHIP (-5)       /* a HIP call failed; see he_last_hip_error */
#define HE_ENODEV (-6)     /* device function called on a host-only context */
#define HE_ENOMEM (-7)
#define HE_ESCRATCH (-8)   /* the operation needs more than the library's static scratch array holds */

typedef struct he_ctx he_ctx;
typedef struct he_sk he_sk;
typedef struct he_evk he_evk;

typedef struct {
    int32_t logN;      /* ring degree N = 2^logN; the device kernels are built for logN = 12, 16 and 17 */
    int32_t L;         /* number of ciphertext primes */
    int32_t K;         /* number of special primes */
    int32_t dnum;      /* number of key-switching digits; alpha = ceil(L/dnum) primes per digit */
    const uint64_t *q; /* [L] */
    const uint64_t *p; /* [K] */
} he_params;

/* ---- context -------------------------------------------------------------------------- */

/* Builds all tables (roots of unity, twiddles, base-conversion constants) on the host and,
 * when device >= 0, uploads them to that HIP device.  device = -1 gives a host-only context on
 * which the host functions work and every device function returns HE_ENODEV.
 * HE_EINVAL: a modulus that is not below 2^60, not = 1 mod 2N or without a 2N-th root of unity, a repeated
 * modulus, dnum < 1; and, for a device context, a size the kernels are not built for: logN other than 12, 16,
 * 17; more than 8 primes per digit (alpha = ceil(L/dnum)) or more than 8 special primes (more than 4 of either
 * at logN = 17); L + K above 64. */
int32_t he_ctx_create(const he_params *params, int32_t device, he_ctx **out);
void he_ctx_destroy(he_ctx *ctx);
const char *he_strerror(int32_t code);
/* Text of the last HIP error seen by this context ("" if none).  Owned by the context. */
const char *he_last_hip_error(const he_ctx *ctx);
/* Modulus i and its 2N-th root of unity psi_i. */
int32_t he_ctx_modulus(const he_ctx *ctx, int32_t i, uint64_t *modulus, uint64_t *psi);
/* Selects the base conversions of every later key switch of this context (Mult, Rotate, their batched and
 * fused forms): exact = 0, the default: the fast conversions (ModUp leaves k D, 0 <= k < digit size, in the
 * raised value; ModDown divides by P up to an integer error below K/2).  exact = 1: the corrected variant, a
 * separately specified form: ModUp takes out v D with v = floor(s), s = sum over the digit's limbs in order of
 * (double)y_i * (1.0 / (double)q_i), so that the raised value is the digit's residue in [0, D); ModDown takes
 * out v P with v = rint(s), s = sum over the centred digits in order of (double)y'_k * (1.0 / (double)p_k), so that
 * the result is u/P rounded to nearest.  Every product and sum of s is one IEEE double operation (no fused
 * multiply-add), rint rounds halves to even; where the exact sum is within the rounding error of s of an
 * integer (a half for ModDown) v may be one off, which changes the result by one source modulus and nothing
 * else.  The paper defers the scheme to the CKKS literature and fixes neither form.  Not thread safe against
 * calls that are being enqueued. */
int32_t he_ctx_set_conversion(he_ctx *ctx, int32_t exact);
/* Galois element 5^r mod 2N of a left rotation by r slots (r may be negative). */
int32_t he_galois_element(const he_ctx *ctx, int32_t r, uint64_t *g);
/* The 38 cumulative thresholds of the discrete Gaussian sampler (sigma 3.2, support [-19,19]). */
int32_t he_gauss_cdt(uint64_t out[38]);
/* Bytes of device workspace that hmult_relin / hrot / hrot_many / rescale / rotate_sum need at
 * `level` for `count` ciphertexts processed by one batched call (1 for the single-ciphertext calls). */
int32_t he_workspace_bytes(const he_ctx *ctx, int32_t level, int32_t count, size_t *out);

/* ---- host: keys, encoding, encryption (the user side; Section 2.2) ----------------------- */

/* Randomness: word i of stream (seed, tag) is mix(key + (i+1)*G), key = mix(mix(seed+G) + tag*G),
 * mix = the SplitMix64 finaliser, G = 0x9E3779B97F4A7C15; tag = kind<<32 | digit<<16 | modulus
 * index, kinds 1 secret, 2 key mask, 3 key error, 4 encryption mask, 5 encryption error.
 * Uniform residues keep the low bitlen(q) bits of a word and reject values >= q; ternary values
 * reject words >= 3*floor(2^64/3) and map word mod 3 = 0,1,2 to 0,+1,-1; Gaussian values are
 * -19 + #{thresholds <= word}. */

/* Ternary secret key. */
int32_t he_keygen_secret(he_ctx *ctx, uint64_t seed, he_sk **out);
/* Secret with exactly h non-zero coefficients (+-1), as bootstrapping wants it: stream kind 11; a position
 * is the low logN bits of a word, redrawn while that position is taken; the next word's low bit is the sign
 * (0: +1).  HE_EINVAL unless 1 <= h <= N. */
int32_t he_keygen_secret_sparse(he_ctx *ctx, uint64_t seed, int32_t h, he_sk **out);
void he_sk_destroy(he_sk *sk);
/* Copies the N secret coefficients (-1, 0, +1). */
int32_t he_sk_coeffs(const he_sk *sk, int8_t *h_out);

/* Switching keys to s: from s^2 (relinearisation) or from sigma_g(s), g = 5^r mod 2N (rotation
 * by r slots).  For digit j and modulus i: a uniform, e Gaussian,
 * b = -a*s + e + (q_i in digit j ? P * s' : 0).  The key is kept on the host and, if the
 * context has a device, uploaded to it. */
int32_t he_keygen_relin(he_ctx *ctx, const he_sk *sk, uint64_t seed, he_evk **out);
int32_t he_keygen_rot(he_ctx *ctx, const he_sk *sk, int32_t r, uint64_t seed, he_evk **out);
/* Key of the automorphism X -> X^(2N-1) = X^-1, which conjugates every slot (slot j sits at a root zeta_j
 * and its conjugate root is zeta_j^-1).  Applied with he_hrot, which applies the automorphism of whatever
 * Galois key it is given. */
int32_t he_keygen_conj(he_ctx *ctx, const he_sk *sk, uint64_t seed, he_evk **out);
/* Public encryption key (b, a), h_pk_out [2][L][N] on the host, NTT domain: a uniform (stream kind 6, one
 * stream per modulus), b = -a s + e with e Gaussian (kind 7).  Section 2.2 lets the data owner encrypt;
 * with this key a party without the secret can do so too. */
int32_t he_keygen_public(const he_ctx *ctx, const he_sk *sk, uint64_t seed, uint64_t *h_pk_out);
/* Public-key encryption of an integer plaintext: c0 = v b + e0 + m, c1 = v a + e1 on the first `level`
 * moduli, v ternary (kind 8), e0, e1 Gaussian (kinds 9, 10).  h_ct_out [2][level][N], NTT domain. */
int32_t he_encrypt_public_coeffs(const he_ctx *ctx, const uint64_t *h_pk, const int64_t *h_coeffs, int32_t level,
                                 uint64_t seed, uint64_t *h_ct_out);
/* Wraps a caller-made key-shaped buffer [dnum][2][L+K][N] (host memory, copied) as a key for the
 * Galois element g (1 = relinearisation): used for throughput runs on synthetic residues. */
int32_t he_evk_from_host(he_ctx *ctx, const uint64_t *h_evk, uint64_t g, he_evk **out);
/* Copies the key to host memory, [dnum][2][L+K][N]. */
int32_t he_evk_to_host(const he_evk *evk, uint64_t *h_out);
void he_evk_destroy(he_evk *evk);

/* Encode: m_k = rint(scale * (2/N) * Re sum_j z_j zeta_j^(-k)), z zero-padded from n_used to N/2
 * slots; h_im may be NULL.  Decode is the inverse map on (centred) coefficients given as doubles. */
int32_t he_encode(const he_ctx *ctx, const double *h_re, const double *h_im, int32_t n_used, double scale,
                  int64_t *h_coeffs_out);
int32_t he_decode(const he_ctx *ctx, const double *h_coeffs, double scale, double *h_re, double *h_im);
/* Integer polynomial -> NTT-domain plaintext [level][N] for he_pmult. */
int32_t he_plain_to_ntt(const he_ctx *ctx, const int64_t *h_coeffs, int32_t level, uint64_t *h_out);
/* Symmetric encryption of an integer polynomial: c1 = a uniform, c0 = -a*s + e + m.  Output
 * [2][level][N] in host memory. */
int32_t he_encrypt_coeffs(const he_ctx *ctx, const he_sk *sk, const int64_t *h_coeffs, int32_t level, uint64_t seed,
                          uint64_t *h_ct_out);
/* c0 + c1*s, inverse NTT, CRT over the first min(level,3) limbs, centred lift -> N doubles. */
int32_t he_decrypt_coeffs(const he_ctx *ctx, const he_sk *sk, const uint64_t *h_ct, int32_t level, double *h_coeffs);
/* he_decrypt_coeffs followed by he_decode; h_re / h_im receive N/2 values (h_im may be NULL). */
int32_t he_decrypt(const he_ctx *ctx, const he_sk *sk, const uint64_t *h_ct, int32_t level, double scale, double *h_re,
                   double *h_im);

/* ---- device: polynomial arithmetic ---------------------------------------------------------- */

/* In-place forward / inverse negacyclic NTT of `batch` limbs stored back to back at d_limbs
 * ([batch][N]); limb b is taken modulo modulus index h_mod_idx[b] (host array, read before
 * return). */
int32_t he_ntt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream);
int32_t he_intt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream);

/* Add / Sub of two level-`level` ciphertexts (Section 2.2, Add).  d_out may alias d_a or d_b. */
int32_t he_add(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level, void *stream);
int32_t he_sub(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level, void *stream);
/* Ciphertext times NTT-domain plaintext [level][N]; d_out may alias d_ct. */
int32_t he_pmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *d_pt, uint64_t *d_out, int32_t level,
                 void *stream);
/* out = sum over k < count of ct_k * pt_k in one pass: h_d_cts / h_d_pts are host arrays of `count` device
 * pointers ([2][level][N] ciphertexts, [level][N] NTT-domain plaintexts), 1 <= count <= 64.  The residues
 * equal those of `count` he_pmult calls summed with he_add.  d_out may alias one of the ciphertexts only
 * if that ciphertext is not read by another term (each output word depends on the same word of every term). */
int32_t he_pmult_sum(he_ctx *ctx, const uint64_t *const *h_d_cts, const uint64_t *const *h_d_pts, int32_t count,
                     uint64_t *d_out, int32_t level, void *stream);
/* Ciphertext times one residue per limb (h_scalar[i] in [0,q_i), host array read before return). */
int32_t he_cmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out, int32_t level,
                 void *stream);

/* Ciphertext plus a plaintext constant given as one residue per limb (h_scalar[i] in [0,q_i)): a
 * constant polynomial has that value at every evaluation point, so it is added to every word of
 * c0.  d_out may alias d_ct. */
int32_t he_add_const(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out, int32_t level,
                     void *stream);
/* Drops limbs: copies the first out_level limbs of both components of a level-in_level
 * ciphertext into d_out [2][out_level][N] (no arithmetic; the scale is unchanged). */
int32_t he_moddrop(he_ctx *ctx, const uint64_t *d_ct, int32_t in_level, uint64_t *d_out, int32_t out_level,
                   void *stream);

/* ---- device: the hot path -------------------------------------------------------------------- */

/* Mult without the rescale (Section 2.2, Mult): tensor product d0 = a0 b0, d1 = a0 b1 + a1 b0,
 * d2 = a1 b1, key switch of d2 with the relinearisation key, out = (d0 + k0, d1 + k1), level
 * unchanged.  d_out [2][level][N] may alias d_a or d_b. */
int32_t he_hmult_relin(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out,
                       int32_t level, void *d_ws, size_t ws_bytes, void *stream);
/* Mult with the rescale that Section 2.2 attaches to it (level l -> l-1), in one call: the residues of
 * he_rescale(he_hmult_relin(a, b)), bit for bit, with one forward transform per output limb instead of two
 * (the ModDown and rescale corrections of a limb are transformed as one polynomial).  d_out is
 * [2][level-1][N] and may alias d_a or d_b; level >= 2 (HE_ELEVEL otherwise).  Workspace as for
 * he_hmult_relin (he_workspace_bytes). */
int32_t he_hmult_relin_rescale(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                               uint64_t *d_out, int32_t level, void *d_ws, size_t ws_bytes, void *stream);
/* Drops the last limb with centred rounding: out[i] = (c[i] - [c_last centred]_{q_i}) / q_last.
 * d_out is [2][level-1][N] and must not alias d_ct. */
int32_t he_rescale(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level, void *d_ws, size_t ws_bytes,
                   void *stream);
/* ModRaise, the first step of Bootstrap (Section 2.2 lists the operation; the construction is the published
 * one): d_ct [2][1][N] modulo q_0 -> d_out [2][level_out][N], the centred coefficients of both components
 * reduced modulo every q_i.  The result decrypts to m + q_0 I with a small integer polynomial I.
 * level_out >= 2; d_out must not alias d_ct; workspace as for level_out. */
int32_t he_modraise(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level_out, void *d_ws, size_t ws_bytes,
                    void *stream);
/* Rotate: the digits of c1 are raised un-rotated, the automorphism sigma_g is applied to the
 * raised digits and to c0, then inner product with the key and ModDown:
 * out = (sigma_g(c0) + k0, k1).  d_out must not alias d_ct. */
int32_t he_hrot(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level, void *d_ws,
                size_t ws_bytes, void *stream);
/* `count` rotations of one ciphertext sharing a single decomposition + ModUp (hoisting);
 * h_d_outs is a host array of `count` device pointers.  Bit-identical to `count` he_hrot calls.
 * The workspace must hold one operation (he_workspace_bytes with count 1); if it holds m >= 2 operations,
 * up to min(m, 32) rotations at a time also share their inner-product, inverse and ModDown launches. */
int32_t he_hrot_many(he_ctx *ctx, const he_evk *const *rots, int32_t count, const uint64_t *d_ct,
                     uint64_t *const *h_d_outs, int32_t level, void *d_ws, size_t ws_bytes, void *stream);
/* for k < count: ct <- ct + Rotate(ct, shift0 * 2^k), in place; rots[k] is the key of that shift. */
int32_t he_rotate_sum(he_ctx *ctx, const he_evk *const *rots, int32_t count, uint64_t *d_ct, int32_t level,
                      void *d_ws, size_t ws_bytes, void *stream);

/* ---- device: a rotation that allocates nothing and takes no workspace ------------------------- */

/* For callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  he_hrot with the library's own scratch
 * array in place of the workspace argument: a file-scope device array of HE_STATIC_SCRATCH_BYTES (64 MiB)
 * that every GPU the library runs on holds until the process ends.  Same result as he_hrot, bit for bit.
 * The call makes no hipMalloc / hipFree and enqueues only kernels on `stream`.  A level whose workspace
 * (he_workspace_bytes(level, 1)) exceeds the array is refused with HE_ESCRATCH before anything is launched:
 * the array holds every level at N = 2^12 and levels up to 9 of the 24-prime, dnum = 6 set at N = 2^16.
 * All calls on one GPU share that GPU's array (whatever the context), which keeps the last call's contents;
 * the operation needs no zeroed memory.  Calls that overlap on one GPU (two streams, two threads) race on it:
 * order them on one stream or with events. */
#define HE_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int32_t he_hrot_noalloc(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                        void *stream);

/* ---- device: batches of independent ciphertexts ----------------------------------------------- */

/* The same operations on `count` ciphertexts stored back to back ([count][2][level][N]), all at
 * the same level and, for key switching, with the same key: every kernel is launched once over
 * the whole batch, which keeps the launches large.  Results are bit-identical to `count` single
 * calls.  The workspace must hold he_workspace_bytes(level, count); count * workspace limbs must
 * stay below 65536 (HE_EINVAL otherwise).  Aliasing rules are those of the single calls. */
int32_t he_add_batch(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                     int32_t count, void *stream);
int32_t he_sub_batch(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                     int32_t count, void *stream);
/* one plaintext [level][N] for the whole batch */
int32_t he_pmult_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *d_pt, uint64_t *d_out, int32_t level,
                       int32_t count, void *stream);
int32_t he_cmult_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out, int32_t level,
                       int32_t count, void *stream);
int32_t he_add_const_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out,
                           int32_t level, int32_t count, void *stream);
int32_t he_moddrop_batch(he_ctx *ctx, const uint64_t *d_ct, int32_t in_level, uint64_t *d_out, int32_t out_level,
                         int32_t count, void *stream);
int32_t he_hmult_relin_batch(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                             uint64_t *d_out, int32_t level, int32_t count, void *d_ws, size_t ws_bytes, void *stream);
/* Batched form of he_hmult_relin_rescale. */
int32_t he_hmult_relin_rescale_batch(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                                     uint64_t *d_out, int32_t level, int32_t count, void *d_ws, size_t ws_bytes,
                                     void *stream);
int32_t he_rescale_batch(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level, int32_t count, void *d_ws,
                         size_t ws_bytes, void *stream);
int32_t he_hrot_batch(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                      int32_t count, void *d_ws, size_t ws_bytes, void *stream);
/* Rotate (Section 2.2) of `count` independent ciphertexts at one level, operation o with its own key rots[o]
 * (host array of key handles; any mix of Galois elements other than 1): the launches of he_hrot_batch with one
 * key per operation.  Bit-identical to he_hrot(rots[o], ct o).  Operations are processed in groups of at most 32;
 * a workspace for fewer operations than that (at least one) makes the groups smaller. */
int32_t he_hrot_batch_keys(he_ctx *ctx, const he_evk *const *rots, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                           int32_t count, void *d_ws, size_t ws_bytes, void *stream);
/* Rotate (Section 2.2) of `count` independent ciphertexts at mixed levels in shared launches: operation o is a
 * level-h_levels[o] ciphertext (host array) with its own key rots[o].  The ciphertexts are packed back to back at
 * d_ct (operation o starts sum_{o' < o} 2 h_levels[o'] limbs in) and the results are packed the same way at
 * d_out, which must not overlap d_ct.  Bit-identical to he_hrot(rots[o], ct o, level h_levels[o]).  Operations
 * are processed in groups of at most 32 that share every launch; a group's buffers are laid out for its largest
 * level, so the workspace must hold at least he_workspace_bytes(largest level, 1) and a workspace of
 * he_workspace_bytes(largest level, 32) gives full groups.  Neighbouring operations with the same key share its
 * memory traffic: sort the operations by key. */
int32_t he_hrot_batch_levels(he_ctx *ctx, const he_evk *const *rots, const int32_t *h_levels, const uint64_t *d_ct,
                             uint64_t *d_out, int32_t count, void *d_ws, size_t ws_bytes, void *stream);
/* n_rot sequential rotate-and-add steps applied to every ciphertext of the batch, in place */
int32_t he_rotate_sum_batch(he_ctx *ctx, const he_evk *const *rots, int32_t n_rot, uint64_t *d_ct, int32_t level,
                            int32_t count, void *d_ws, size_t ws_bytes, void *stream);

/* ---- measurement ------------------------------------------------------------------------- */

/* Per-kernel timing for benchmarks: between start and stop every kernel the library launches is
 * bracketed by a pair of HIP events on its stream.  Stop waits for the recorded events and fills
 * `out` with one entry per kernel that ran: launch count, summed duration, and the summed bytes
 * each launch has to move by the definition of its step (inputs read once + outputs written
 * once).  Not thread safe; keep it off in production paths. */
typedef struct {
    char name[48];
    int64_t launches;
    double total_ms;
    double bytes;
} he_kernel_stat;
int32_t he_profile_start(he_ctx *ctx);
/* *n_out receives the number of kernels that ran; at most max_out entries are written, and HE_EINVAL is returned
 * (with the first max_out entries filled and *n_out set to the number needed) when max_out is too small. */
int32_t he_profile_stop(he_ctx *ctx, he_kernel_stat *out, int32_t max_out, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* HE_H_ */
