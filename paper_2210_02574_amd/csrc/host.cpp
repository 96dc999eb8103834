// Host side of the RNS-CKKS library: context tables, the counter-based generator and samplers,
// encoding, key generation, encryption and decryption (the user side of the protocol in the
// paper's Section 2.2 and Figure 1).  Arithmetic here uses Shoup-form constants and lazy
// butterflies, the same formulation as the device kernels.
#include <algorithm>
#include <cmath>
#include <atomic>
#include <complex>
#include <cstring>
#include <functional>
#include <new>
#include <thread>

#include "he_internal.h"

namespace hostmath {

u64 mul_mod(u64 a, u64 b, u64 q) { return (u64)((u128)a * b % q); }

u64 pow_mod(u64 b, u64 e, u64 q)
{
    u64 r = 1;
    b %= q;
    for (; e; e >>= 1) {
        if (e & 1) r = mul_mod(r, b, q);
        b = mul_mod(b, b, q);
    }
    return r;
}

u64 inv_mod(u64 a, u64 q) { return pow_mod(a % q, q - 2, q); }

ShoupConst shoup(u64 w, u64 q)
{
    ShoupConst s;
    s.w = w;
    s.wp = (u64)(((u128)w << 64) / q);
    return s;
}

static inline u64 mul_hi(u64 a, u64 b) { return (u64)(((u128)a * b) >> 64); }
// w*x mod q up to one extra q: result in [0, 2q) for any 64-bit x
static inline u64 mul_shoup_lazy(u64 x, ShoupConst w, u64 q) { return x * w.w - mul_hi(x, w.wp) * q; }
static inline u64 mul_shoup(u64 x, ShoupConst w, u64 q)
{
    u64 r = mul_shoup_lazy(x, w, q);
    return r >= q ? r - q : r;
}

u64 least_primitive_root(u64 q)
{
    std::vector<u64> fac;
    u64 m = q - 1;
    for (u64 f = 2; f * f <= m; f += (f == 2 ? 1 : 2))
        if (m % f == 0) {
            fac.push_back(f);
            while (m % f == 0) m /= f;
        }
    if (m > 1) fac.push_back(m);
    for (u64 g = 2; g < q; g++) {
        bool ok = true;
        for (u64 f : fac)
            if (pow_mod(g, (q - 1) / f, q) == 1) {
                ok = false;
                break;
            }
        if (ok) return g;
    }
    return 0;
}

unsigned bit_reverse(unsigned x, int bits)
{
    unsigned r = 0;
    for (int i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

void ntt(const he_ctx *c, int mi, u64 *a)
{
    const u64 N = c->N, q = c->mod[mi], q2 = 2 * q;
    const ShoupConst *tw = c->tw_fwd.data() + (size_t)mi * N;
    for (u64 m = 1, t = N >> 1; m < N; m <<= 1, t >>= 1)
        for (u64 i = 0; i < m; i++) {
            const ShoupConst W = tw[m + i];
            u64 *x = a + 2 * i * t, *y = x + t;
            for (u64 j = 0; j < t; j++) {
                u64 u = x[j];
                if (u >= q2) u -= q2;
                u64 v = mul_shoup_lazy(y[j], W, q);
                x[j] = u + v;
                y[j] = u - v + q2;
            }
        }
    for (u64 j = 0; j < N; j++) {
        u64 v = a[j];
        if (v >= q2) v -= q2;
        if (v >= q) v -= q;
        a[j] = v;
    }
}

void intt(const he_ctx *c, int mi, u64 *a)
{
    const u64 N = c->N, q = c->mod[mi], q2 = 2 * q;
    const ShoupConst *tw = c->tw_inv.data() + (size_t)mi * N;
    for (u64 m = N >> 1, t = 1; m >= 1; m >>= 1, t <<= 1)
        for (u64 i = 0; i < m; i++) {
            const ShoupConst W = tw[m + i];
            u64 *x = a + 2 * i * t, *y = x + t;
            for (u64 j = 0; j < t; j++) {
                u64 u = x[j], v = y[j];
                u64 s = u + v;
                if (s >= q2) s -= q2;
                x[j] = s;
                y[j] = mul_shoup_lazy(u - v + q2, W, q);
            }
        }
    const ShoupConst ni = c->ninv[(size_t)mi * 2];
    for (u64 j = 0; j < N; j++) a[j] = mul_shoup(a[j], ni, q);
}

void parallel_for(int n, const std::function<void(int)> &f)
{
    int nt = (int)std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
    nt = std::min(nt, n);
    if (nt <= 1) {
        for (int i = 0; i < n; i++) f(i);
        return;
    }
    std::vector<std::thread> th;
    for (int t = 0; t < nt; t++)
        th.emplace_back([=, &f]() {
            for (int i = t; i < n; i += nt) f(i);
        });
    for (auto &x : th) x.join();
}

} // namespace hostmath

using namespace hostmath;

// ------------------------------------------------------------------------------------- context

static const u64 kGaussCdt[38] = {
#include "gauss_cdt.inc"
};

extern "C" const char *he_strerror(int32_t code)
{
    switch (code) {
    case HE_OK: return "ok";
    case HE_EINVAL: return "invalid argument";
    case HE_ELEVEL: return "level out of range";
    case HE_ENOKEY: return "missing or mismatched key";
    case HE_EWORKSPACE: return "workspace too small";
    case HE_EHIP: return "HIP error";
    case HE_ENODEV: return "context has no device";
    case HE_ENOMEM: return "out of memory";
    case HE_ESCRATCH: return "operation does not fit the static scratch array";
    }
    return "unknown error";
}

extern "C" const char *he_last_hip_error(const he_ctx *ctx) { return ctx ? ctx->hip_err.c_str() : ""; }

extern "C" int32_t he_gauss_cdt(uint64_t out[38])
{
    if (!out) return HE_EINVAL;
    memcpy(out, kGaussCdt, sizeof(kGaussCdt));
    return HE_OK;
}

static u64 prod_mod_excluding(const std::vector<u64> &ms, int lo, int hi, int skip, u64 t)
{
    u64 r = 1 % t;
    for (int i = lo; i < hi; i++)
        if (i != skip) r = mul_mod(r, ms[i] % t, t);
    return r;
}

extern "C" int32_t he_ctx_create(const he_params *p, int32_t device, he_ctx **out)
{
    if (!p || !out || !p->q || !p->p) return HE_EINVAL;
    if (p->logN < 2 || p->logN > 17 || p->L < 1 || p->K < 1 || p->dnum < 1 || p->dnum > p->L) return HE_EINVAL;
    if (p->L + p->K > 255) return HE_EINVAL;
    he_ctx *c = new (std::nothrow) he_ctx;
    if (!c) return HE_ENOMEM;
    c->logN = p->logN;
    c->N = (u64)1 << p->logN;
    c->L = p->L;
    c->K = p->K;
    c->dnum = p->dnum;
    c->alpha = (p->L + p->dnum - 1) / p->dnum;
    c->M = p->L + p->K;
    c->device = -1;
    const u64 N = c->N;
    const int M = c->M, L = c->L, K = c->K, alpha = c->alpha;
    for (int i = 0; i < M; i++) {
        u64 t = i < L ? p->q[i] : p->p[i - L];
        if (t >= ((u64)1 << 60) || t < 2 * N || (t - 1) % (2 * N) != 0) {
            delete c;
            return HE_EINVAL;
        }
        for (int i2 = 0; i2 < i; i2++)
            if (c->mod[i2] == t) {
                delete c;
                return HE_EINVAL;
            }
        c->mod.push_back(t);
    }
    try {
        c->psi.resize(M);
        c->modc.resize(M);
        c->tw_fwd.resize((size_t)M * N);
        c->tw_inv.resize((size_t)M * N);
        c->ninv.resize((size_t)M * 2);
        c->twd_fwd.assign((size_t)M * N, 0.0);
        c->twd_inv.assign((size_t)M * N, 0.0);
        c->ninvd.assign((size_t)M * 2, 0.0);
    } catch (...) {
        delete c;
        return HE_ENOMEM;
    }
    std::atomic<bool> bad(false); // written by several workers
    parallel_for(M, [&](int i) {
        const u64 t = c->mod[i];
        const u64 g = least_primitive_root(t);
        const u64 psi = pow_mod(g, (t - 1) / (2 * N), t);
        if (g == 0 || pow_mod(psi, N, t) != t - 1) {
            bad = true; // not a prime with a 2N-th root of unity
            return;
        }
        const u64 ipsi = inv_mod(psi, t);
        c->psi[i] = psi;
        c->modc[i].q = t;
        c->modc[i].one_p = (u64)((((u128)1) << 64) / t);
        c->modc[i].r = shoup((u64)((((u128)1) << 64) % t), t);
        // powers in natural order, stored at the bit-reversed position
        u64 pw = 1, ipw = 1;
        for (u64 e = 0; e < N; e++) {
            const size_t pos = (size_t)i * N + bit_reverse((unsigned)e, c->logN);
            c->tw_fwd[pos] = shoup(pw, t);
            c->tw_inv[pos] = shoup(ipw, t);
            pw = mul_mod(pw, psi, t);
            ipw = mul_mod(ipw, ipsi, t);
        }
        const u64 ni = inv_mod(N % t, t);
        c->ninv[(size_t)i * 2 + 0] = shoup(ni, t);
        c->ninv[(size_t)i * 2 + 1] = shoup(mul_mod(ni, c->tw_inv[(size_t)i * N + 1].w, t), t);
        c->modc[i].qd = 0.0;
        c->modc[i].qinvd = 0.0;
        if (t < ((u64)1 << 50)) {
            // balanced representatives as doubles for the FP64 butterflies
            auto bal = [t](u64 w) { return w > t / 2 ? -(double)(t - w) : (double)w; };
            c->modc[i].qd = (double)t;
            c->modc[i].qinvd = 1.0 / (double)t;
            for (u64 e = 0; e < N; e++) {
                c->twd_fwd[(size_t)i * N + e] = bal(c->tw_fwd[(size_t)i * N + e].w);
                c->twd_inv[(size_t)i * N + e] = bal(c->tw_inv[(size_t)i * N + e].w);
            }
            c->ninvd[(size_t)i * 2 + 0] = bal(c->ninv[(size_t)i * 2 + 0].w);
            c->ninvd[(size_t)i * 2 + 1] = bal(c->ninv[(size_t)i * 2 + 1].w);
        }
    });
    if (bad) {
        delete c;
        return HE_EINVAL;
    }
    // ModUp constants: digit j with a active limbs -> slot j*alpha + (a-1)
    c->up_inv.assign((size_t)c->dnum * alpha * alpha, ShoupConst{0, 0});
    c->up_hat.assign((size_t)c->dnum * alpha * alpha * M, 0);
    for (int j = 0; j < c->dnum; j++)
        for (int a = 1; a <= alpha; a++) {
            const int lo = j * alpha, hi = lo + a;
            if (hi > L) break;
            const size_t slot = (size_t)j * alpha + (a - 1);
            for (int ii = 0; ii < a; ii++) {
                const u64 qi = c->mod[lo + ii];
                c->up_inv[slot * alpha + ii] = shoup(inv_mod(prod_mod_excluding(c->mod, lo, hi, lo + ii, qi), qi), qi);
                for (int m = 0; m < M; m++)
                    c->up_hat[(slot * alpha + ii) * M + m] = prod_mod_excluding(c->mod, lo, hi, lo + ii, c->mod[m]);
            }
        }
    // ModDown constants
    c->dn_inv.resize(K);
    c->dn_hat.resize((size_t)K * L);
    c->dn_pinv.resize(L);
    for (int k = 0; k < K; k++) {
        const u64 pk = c->mod[L + k];
        c->dn_inv[k] = shoup(inv_mod(prod_mod_excluding(c->mod, L, M, L + k, pk), pk), pk);
        for (int i = 0; i < L; i++) c->dn_hat[(size_t)k * L + i] = prod_mod_excluding(c->mod, L, M, L + k, c->mod[i]);
    }
    for (int i = 0; i < L; i++) {
        const u64 qi = c->mod[i];
        c->dn_pinv[i] = shoup(inv_mod(prod_mod_excluding(c->mod, L, M, -1, qi), qi), qi);
    }
    // Rescale constants
    c->rs_inv.assign((size_t)L * L, ShoupConst{0, 0});
    for (int l = 0; l < L; l++)
        for (int i = 0; i < L; i++)
            if (i != l) c->rs_inv[(size_t)l * L + i] = shoup(inv_mod(c->mod[l] % c->mod[i], c->mod[i]), c->mod[i]);
    c->rsp_inv.assign((size_t)L * L, ShoupConst{0, 0});
    for (int l = 0; l < L; l++)
        for (int i = 0; i < L; i++)
            if (i != l)
                c->rsp_inv[(size_t)l * L + i] =
                    shoup(mul_mod(c->rs_inv[(size_t)l * L + i].w, c->dn_pinv[i].w, c->mod[i]), c->mod[i]);
    // balanced-double images of the conversion constants for moduli below 2^50
    {
        const u64 kFp = (u64)1 << 50;
        auto bal = [](u64 w, u64 t) { return w > t / 2 ? -(double)(t - w) : (double)w; };
        for (int i = 0; i < L; i++) c->up_split = c->up_split || c->mod[i] >= kFp;
        for (int k = 0; k < K; k++) c->dn_split = c->dn_split || c->mod[L + k] >= kFp;
        c->up_inv_d.assign(c->up_inv.size(), 0.0);
        c->up_hat_d.assign(c->up_hat.size(), 0.0);
        c->up_hat_dh.assign(c->up_hat.size(), 0.0);
        c->up_hat_p.assign(c->up_hat.size(), 0);
        for (size_t e = 0; e < c->up_hat.size(); e++) c->up_hat_p[e] = shoup(c->up_hat[e], c->mod[e % M]).wp;
        c->rq.assign(M, 0.0);
        for (int m = 0; m < M; m++) c->rq[m] = 1.0 / (double)c->mod[m];
        c->up_dmod.assign((size_t)c->dnum * alpha * M, 0);
        c->up_dmod_d.assign(c->up_dmod.size(), 0.0);
        for (int j = 0; j < c->dnum; j++)
            for (int a = 1; a <= alpha; a++) {
                const int lo = j * alpha;
                if (lo + a > L) break;
                const size_t slot = (size_t)j * alpha + (a - 1);
                for (int m = 0; m < M; m++) { // D = product of the digit's a active primes, modulo every modulus
                    const u64 t = c->mod[m];
                    u64 d = 1;
                    for (int ii = 0; ii < a; ii++) d = mul_mod(d, c->mod[lo + ii] % t, t);
                    c->up_dmod[slot * M + m] = d;
                    if (t < kFp) c->up_dmod_d[slot * M + m] = bal(d, t);
                }
                for (int ii = 0; ii < a; ii++) {
                    const u64 qi = c->mod[lo + ii];
                    if (qi < kFp) c->up_inv_d[slot * alpha + ii] = bal(c->up_inv[slot * alpha + ii].w, qi);
                    for (int m = 0; m < M; m++) {
                        const u64 t = c->mod[m];
                        if (t >= kFp) continue;
                        const u64 h = c->up_hat[(slot * alpha + ii) * M + m];
                        c->up_hat_d[(slot * alpha + ii) * M + m] = bal(h, t);
                        c->up_hat_dh[(slot * alpha + ii) * M + m] = bal(mul_mod(h, ((u64)1 << 31) % t, t), t);
                    }
                }
            }
        c->dn_inv_d.assign(K, 0.0);
        c->dn_hat_d.assign((size_t)K * L, 0.0);
        c->dn_hat_dh.assign((size_t)K * L, 0.0);
        c->dn_pinv_d.assign(L, 0.0);
        c->dn_pmod.assign(L, 0);
        c->dn_pmod_d.assign(L, 0.0);
        for (int i = 0; i < L; i++) c->dn_pmod[i] = prod_mod_excluding(c->mod, L, M, -1, c->mod[i]);
        c->dn_r50_d.assign(L, 0.0);
        c->dn_fold = c->dn_split;
        for (int i = 0; i < L; i++) {
            const u64 t = c->mod[i];
            if (t >= kFp) continue;
            c->dn_r50_d[i] = bal(kFp % t, t);
            if (std::fabs(c->dn_r50_d[i]) >= 1099511627776.0) c->dn_fold = false; // 2^40
        }
        c->rs_inv_d.assign((size_t)L * L, 0.0);
        c->rsp_inv_d.assign((size_t)L * L, 0.0);
        for (int k = 0; k < K; k++) {
            if (c->mod[L + k] < kFp) c->dn_inv_d[k] = bal(c->dn_inv[k].w, c->mod[L + k]);
            for (int i = 0; i < L; i++) {
                const u64 t = c->mod[i];
                if (t >= kFp) continue;
                const u64 h = c->dn_hat[(size_t)k * L + i];
                c->dn_hat_d[(size_t)k * L + i] = bal(h, t);
                c->dn_hat_dh[(size_t)k * L + i] = bal(mul_mod(h, ((u64)1 << 31) % t, t), t);
            }
        }
        for (int i = 0; i < L; i++) {
            const u64 t = c->mod[i];
            if (t >= kFp) continue;
            c->dn_pinv_d[i] = bal(c->dn_pinv[i].w, t);
            c->dn_pmod_d[i] = bal(c->dn_pmod[i], t);
            for (int l = 0; l < L; l++)
                if (l != i) {
                    c->rs_inv_d[(size_t)l * L + i] = bal(c->rs_inv[(size_t)l * L + i].w, t);
                    c->rsp_inv_d[(size_t)l * L + i] = bal(c->rsp_inv[(size_t)l * L + i].w, t);
                }
        }
    }
    // encode/decode tables
    c->root_re.resize(2 * N);
    c->root_im.resize(2 * N);
    for (u64 e = 0; e < 2 * N; e++) {
        c->root_re[e] = std::cos(M_PI * (double)e / (double)N);
        c->root_im[e] = std::sin(M_PI * (double)e / (double)N);
    }
    c->slot_exp.resize(N / 2);
    u64 g5 = 1;
    for (u64 j = 0; j < N / 2; j++) {
        c->slot_exp[j] = (uint32_t)g5;
        g5 = (g5 * 5) % (2 * N);
    }
    if (device >= 0) {
        c->device = device;
        int32_t rc = dev_upload_tables(c);
        if (rc != HE_OK) {
            // keep the error text reachable: the caller gets no context, so print nothing and fail
            dev_free_tables(c);
            delete c;
            return rc;
        }
    }
    *out = c;
    return HE_OK;
}

extern "C" void he_ctx_destroy(he_ctx *ctx)
{
    if (!ctx) return;
    dev_free_tables(ctx);
    delete ctx;
}

extern "C" int32_t he_ctx_modulus(const he_ctx *ctx, int32_t i, uint64_t *modulus, uint64_t *psi)
{
    if (!ctx || i < 0 || i >= ctx->M) return HE_EINVAL;
    if (modulus) *modulus = ctx->mod[i];
    if (psi) *psi = ctx->psi[i];
    return HE_OK;
}

extern "C" int32_t he_ctx_set_conversion(he_ctx *ctx, int32_t exact)
{
    if (!ctx || (exact != 0 && exact != 1)) return HE_EINVAL;
    ctx->exact_conv = exact;
    return HE_OK;
}

extern "C" int32_t he_galois_element(const he_ctx *ctx, int32_t r, uint64_t *g)
{
    if (!ctx || !g) return HE_EINVAL;
    const int64_t n = (int64_t)(ctx->N / 2);
    int64_t rr = r % n;
    if (rr < 0) rr += n;
    *g = ctx->slot_exp[(size_t)rr];
    return HE_OK;
}

// ---------------------------------------------------------------------------------- randomness

static const u64 kGamma = 0x9E3779B97F4A7C15ull;
static inline u64 mix(u64 z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

struct Stream {
    u64 key, ctr;
    Stream(u64 seed, u64 kind, u64 digit, u64 modidx)
    {
        const u64 tag = (kind << 32) | (digit << 16) | modidx;
        key = mix(mix(seed + kGamma) + tag * kGamma);
        ctr = 0;
    }
    u64 next() { return mix(key + (++ctr) * kGamma); }
};

static void sample_uniform(Stream st, u64 q, u64 *out, u64 n)
{
    const int bits = 64 - __builtin_clzll(q);
    const u64 mask = bits == 64 ? ~(u64)0 : (((u64)1 << bits) - 1);
    for (u64 k = 0; k < n; k++) {
        u64 v;
        do v = st.next() & mask;
        while (v >= q);
        out[k] = v;
    }
}

static void sample_ternary(Stream st, int8_t *out, u64 n)
{
    const u64 lim = 3 * (~(u64)0 / 3);
    static const int8_t map[3] = {0, 1, -1};
    for (u64 k = 0; k < n; k++) {
        u64 v;
        do v = st.next();
        while (v >= lim);
        out[k] = map[v % 3];
    }
}

static void sample_gauss(Stream st, int8_t *out, u64 n)
{
    for (u64 k = 0; k < n; k++) {
        const u64 u = st.next();
        // thresholds are sorted: the count of thresholds <= u is an upper bound search
        const int cnt = (int)(std::upper_bound(kGaussCdt, kGaussCdt + 38, u) - kGaussCdt);
        out[k] = (int8_t)(cnt - 19);
    }
}

static inline u64 signed_residue(int64_t v, u64 q)
{
    if (v >= 0) return (u64)v % q;
    const u64 a = ((u64)(-(v + 1)) + 1) % q;
    return a ? q - a : 0;
}

static void small_to_ntt(const he_ctx *c, int mi, const int8_t *s, u64 *out)
{
    const u64 q = c->mod[mi];
    for (u64 j = 0; j < c->N; j++) out[j] = s[j] >= 0 ? (u64)s[j] : q - (u64)(-s[j]);
    ntt(c, mi, out);
}

// ---------------------------------------------------------------------------------------- keys

extern "C" int32_t he_keygen_secret(he_ctx *ctx, uint64_t seed, he_sk **out)
{
    if (!ctx || !out) return HE_EINVAL;
    he_sk *sk = new (std::nothrow) he_sk;
    if (!sk) return HE_ENOMEM;
    sk->ctx = ctx;
    sk->s.resize(ctx->N);
    sk->s_ntt.resize((size_t)ctx->M * ctx->N);
    sample_ternary(Stream(seed, 1, 0, 0), sk->s.data(), ctx->N);
    parallel_for(ctx->M, [&](int i) { small_to_ntt(ctx, i, sk->s.data(), sk->s_ntt.data() + (size_t)i * ctx->N); });
    *out = sk;
    return HE_OK;
}

extern "C" int32_t he_keygen_secret_sparse(he_ctx *ctx, uint64_t seed, int32_t h, he_sk **out)
{
    if (!ctx || !out || h < 1 || (u64)h > ctx->N) return HE_EINVAL;
    he_sk *sk = new (std::nothrow) he_sk;
    if (!sk) return HE_ENOMEM;
    sk->ctx = ctx;
    sk->s.assign(ctx->N, 0);
    sk->s_ntt.resize((size_t)ctx->M * ctx->N);
    Stream st(seed, 11, 0, 0);
    for (int placed = 0; placed < h;) {
        const u64 pos = st.next() & (ctx->N - 1);
        if (sk->s[pos] != 0) continue;
        sk->s[pos] = (st.next() & 1) == 0 ? 1 : -1;
        placed++;
    }
    parallel_for(ctx->M, [&](int i) { small_to_ntt(ctx, i, sk->s.data(), sk->s_ntt.data() + (size_t)i * ctx->N); });
    *out = sk;
    return HE_OK;
}

extern "C" void he_sk_destroy(he_sk *sk) { delete sk; }

extern "C" int32_t he_sk_coeffs(const he_sk *sk, int8_t *h_out)
{
    if (!sk || !h_out) return HE_EINVAL;
    memcpy(h_out, sk->s.data(), sk->s.size());
    return HE_OK;
}

// sp_ntt: s' in NTT form on the L ciphertext moduli
static int32_t make_switch_key(he_ctx *ctx, const he_sk *sk, const std::vector<u64> &sp_ntt, u64 galois, u64 seed,
                               he_evk **out)
{
    const u64 N = ctx->N;
    const int M = ctx->M, L = ctx->L, K = ctx->K;
    he_evk *k = new (std::nothrow) he_evk;
    if (!k) return HE_ENOMEM;
    k->ctx = ctx;
    k->galois = galois;
    try {
        k->host.resize((size_t)ctx->dnum * 2 * M * N);
    } catch (...) {
        delete k;
        return HE_ENOMEM;
    }
    for (int j = 0; j < ctx->dnum; j++) {
        std::vector<int8_t> e(N);
        sample_gauss(Stream(seed, 3, (u64)j, 0), e.data(), N);
        parallel_for(M, [&](int i) {
            const u64 t = ctx->mod[i];
            u64 *b = k->host.data() + (((size_t)j * 2 + 0) * M + i) * N;
            u64 *a = k->host.data() + (((size_t)j * 2 + 1) * M + i) * N;
            sample_uniform(Stream(seed, 2, (u64)j, (u64)i), t, a, N);
            small_to_ntt(ctx, i, e.data(), b);
            const u64 *s = sk->s_ntt.data() + (size_t)i * N;
            const bool in_digit = i < L && i / ctx->alpha == j;
            ShoupConst Pm{0, 0};
            if (in_digit) Pm = shoup(prod_mod_excluding(ctx->mod, L, L + K, -1, t), t);
            const u64 *sp = in_digit ? sp_ntt.data() + (size_t)i * N : nullptr;
            for (u64 x = 0; x < N; x++) {
                u64 v = b[x] + t - mul_mod(a[x], s[x], t);
                if (in_digit) v += mul_shoup(sp[x], Pm, t);
                v %= t;
                b[x] = v;
            }
        });
    }
    if (ctx->device >= 0) {
        int32_t rc = dev_upload_evk(k);
        if (rc != HE_OK) {
            delete k;
            return rc;
        }
        std::vector<u64>().swap(k->host);
    }
    *out = k;
    return HE_OK;
}

extern "C" int32_t he_keygen_relin(he_ctx *ctx, const he_sk *sk, uint64_t seed, he_evk **out)
{
    if (!ctx || !sk || !out || sk->ctx != ctx) return HE_EINVAL;
    const u64 N = ctx->N;
    std::vector<u64> sp((size_t)ctx->L * N);
    parallel_for(ctx->L, [&](int i) {
        const u64 *s = sk->s_ntt.data() + (size_t)i * N;
        for (u64 x = 0; x < N; x++) sp[(size_t)i * N + x] = mul_mod(s[x], s[x], ctx->mod[i]);
    });
    return make_switch_key(ctx, sk, sp, 1, seed, out);
}

// switching key from sigma_g(s) to s
static int32_t make_galois_key(he_ctx *ctx, const he_sk *sk, u64 g, u64 seed, he_evk **out)
{
    const u64 N = ctx->N;
    // sigma_g(s): coefficient j moves to j*g mod 2N, negated when it wraps past N
    std::vector<int8_t> sg(N);
    for (u64 j = 0; j < N; j++) {
        const u64 e = (j * g) & (2 * N - 1);
        if (e < N)
            sg[e] = sk->s[j];
        else
            sg[e - N] = (int8_t)-sk->s[j];
    }
    std::vector<u64> sp((size_t)ctx->L * N);
    parallel_for(ctx->L, [&](int i) { small_to_ntt(ctx, i, sg.data(), sp.data() + (size_t)i * N); });
    return make_switch_key(ctx, sk, sp, g, seed, out);
}

extern "C" int32_t he_keygen_rot(he_ctx *ctx, const he_sk *sk, int32_t r, uint64_t seed, he_evk **out)
{
    if (!ctx || !sk || !out || sk->ctx != ctx) return HE_EINVAL;
    u64 g;
    he_galois_element(ctx, r, &g);
    if (g == 1) return HE_EINVAL; // rotation by a multiple of N/2 needs no key
    return make_galois_key(ctx, sk, g, seed, out);
}

extern "C" int32_t he_keygen_conj(he_ctx *ctx, const he_sk *sk, uint64_t seed, he_evk **out)
{
    if (!ctx || !sk || !out || sk->ctx != ctx) return HE_EINVAL;
    return make_galois_key(ctx, sk, 2 * ctx->N - 1, seed, out);
}

extern "C" int32_t he_evk_from_host(he_ctx *ctx, const uint64_t *h_evk, uint64_t g, he_evk **out)
{
    if (!ctx || !h_evk || !out || !(g & 1) || g >= 2 * ctx->N) return HE_EINVAL;
    he_evk *k = new (std::nothrow) he_evk;
    if (!k) return HE_ENOMEM;
    k->ctx = ctx;
    k->galois = g;
    const size_t words = (size_t)ctx->dnum * 2 * ctx->M * ctx->N;
    try {
        k->host.assign(h_evk, h_evk + words);
    } catch (...) {
        delete k;
        return HE_ENOMEM;
    }
    if (ctx->device >= 0) {
        int32_t rc = dev_upload_evk(k);
        if (rc != HE_OK) {
            delete k;
            return rc;
        }
        std::vector<u64>().swap(k->host);
    }
    *out = k;
    return HE_OK;
}

extern "C" void he_evk_destroy(he_evk *evk)
{
    if (!evk) return;
    dev_free_evk(evk);
    delete evk;
}

// --------------------------------------------------------------------------- encode / decode

typedef std::complex<double> cplx;

// in-place radix-2 FFT of size N: X[k] = sum_u x[u] * exp(sign * 2 pi i u k / N)
static void fft(const he_ctx *c, std::vector<cplx> &x, int sign)
{
    const size_t N = x.size();
    const int lg = c->logN;
    for (size_t i = 0; i < N; i++) {
        size_t j = bit_reverse((unsigned)i, lg);
        if (j > i) std::swap(x[i], x[j]);
    }
    for (size_t len = 2; len <= N; len <<= 1) {
        const size_t half = len >> 1, step = N / len; // root index step in units of exp(2 pi i / N)
        for (size_t s = 0; s < N; s += len)
            for (size_t k = 0; k < half; k++) {
                const size_t e = 2 * k * step; // exponent of exp(i pi / N)
                const cplx w(c->root_re[e], sign * c->root_im[e]);
                const cplx u = x[s + k], v = x[s + k + half] * w;
                x[s + k] = u + v;
                x[s + k + half] = u - v;
            }
    }
}

extern "C" int32_t he_encode(const he_ctx *ctx, const double *h_re, const double *h_im, int32_t n_used, double scale,
                             int64_t *h_coeffs_out)
{
    if (!ctx || !h_re || !h_coeffs_out || n_used < 0 || (u64)n_used > ctx->N / 2 || !(scale > 0)) return HE_EINVAL;
    const u64 N = ctx->N;
    // values at the odd powers zeta^(2u+1): slot j at 5^j, its conjugate at -5^j
    std::vector<cplx> B(N, cplx(0, 0));
    for (int32_t j = 0; j < n_used; j++) {
        const u64 e = ctx->slot_exp[j];
        const cplx z(h_re[j], h_im ? h_im[j] : 0.0);
        B[(e - 1) >> 1] = z;
        B[(2 * N - e - 1) >> 1] = std::conj(z);
    }
    fft(ctx, B, -1);
    for (u64 k = 0; k < N; k++) {
        const cplx tw(ctx->root_re[k], -ctx->root_im[k]);
        const double v = (B[k] * tw).real() * (scale / (double)N);
        if (!(std::fabs(v) < 9.0e18)) return HE_EINVAL;
        h_coeffs_out[k] = (int64_t)std::rint(v);
    }
    return HE_OK;
}

extern "C" int32_t he_decode(const he_ctx *ctx, const double *h_coeffs, double scale, double *h_re, double *h_im)
{
    if (!ctx || !h_coeffs || !h_re || !(scale > 0)) return HE_EINVAL;
    const u64 N = ctx->N;
    std::vector<cplx> Y(N);
    for (u64 k = 0; k < N; k++) Y[k] = h_coeffs[k] * cplx(ctx->root_re[k], ctx->root_im[k]);
    fft(ctx, Y, +1);
    for (u64 j = 0; j < N / 2; j++) {
        const cplx z = Y[(ctx->slot_exp[j] - 1) >> 1] / scale;
        h_re[j] = z.real();
        if (h_im) h_im[j] = z.imag();
    }
    return HE_OK;
}

extern "C" int32_t he_plain_to_ntt(const he_ctx *ctx, const int64_t *h_coeffs, int32_t level, uint64_t *h_out)
{
    if (!ctx || !h_coeffs || !h_out) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    const u64 N = ctx->N;
    parallel_for(level, [&](int i) {
        u64 *o = h_out + (size_t)i * N;
        for (u64 x = 0; x < N; x++) o[x] = signed_residue(h_coeffs[x], ctx->mod[i]);
        ntt(ctx, i, o);
    });
    return HE_OK;
}

// ------------------------------------------------------------------------ encrypt / decrypt

extern "C" int32_t he_encrypt_coeffs(const he_ctx *ctx, const he_sk *sk, const int64_t *h_coeffs, int32_t level,
                                     uint64_t seed, uint64_t *h_ct_out)
{
    if (!ctx || !sk || !h_coeffs || !h_ct_out || sk->ctx != ctx) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    const u64 N = ctx->N;
    std::vector<int8_t> e(N);
    sample_gauss(Stream(seed, 5, 0, 0), e.data(), N);
    parallel_for(level, [&](int i) {
        const u64 t = ctx->mod[i];
        u64 *c0 = h_ct_out + ((size_t)0 * level + i) * N;
        u64 *c1 = h_ct_out + ((size_t)1 * level + i) * N;
        sample_uniform(Stream(seed, 4, 0, (u64)i), t, c1, N);
        // e + m has small coefficients next to q: one transform serves both terms
        for (u64 x = 0; x < N; x++) c0[x] = signed_residue(h_coeffs[x] + (int64_t)e[x], t);
        ntt(ctx, i, c0);
        const u64 *s = sk->s_ntt.data() + (size_t)i * N;
        for (u64 x = 0; x < N; x++) {
            u64 v = c0[x] + t - mul_mod(c1[x], s[x], t);
            c0[x] = v >= t ? v - t : v;
        }
    });
    return HE_OK;
}

extern "C" int32_t he_keygen_public(const he_ctx *ctx, const he_sk *sk, uint64_t seed, uint64_t *h_pk_out)
{
    if (!ctx || !sk || !h_pk_out || sk->ctx != ctx) return HE_EINVAL;
    const u64 N = ctx->N;
    const int L = ctx->L;
    std::vector<int8_t> e(N);
    sample_gauss(Stream(seed, 7, 0, 0), e.data(), N);
    parallel_for(L, [&](int i) {
        const u64 t = ctx->mod[i];
        u64 *b = h_pk_out + ((size_t)0 * L + i) * N;
        u64 *a = h_pk_out + ((size_t)1 * L + i) * N;
        sample_uniform(Stream(seed, 6, 0, (u64)i), t, a, N);
        small_to_ntt(ctx, i, e.data(), b);
        const u64 *s = sk->s_ntt.data() + (size_t)i * N;
        for (u64 x = 0; x < N; x++) {
            const u64 v = b[x] + t - mul_mod(a[x], s[x], t);
            b[x] = v >= t ? v - t : v;
        }
    });
    return HE_OK;
}

extern "C" int32_t he_encrypt_public_coeffs(const he_ctx *ctx, const uint64_t *h_pk, const int64_t *h_coeffs,
                                            int32_t level, uint64_t seed, uint64_t *h_ct_out)
{
    if (!ctx || !h_pk || !h_coeffs || !h_ct_out) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    const u64 N = ctx->N;
    const int L = ctx->L;
    std::vector<int8_t> v(N), e0(N), e1(N);
    sample_ternary(Stream(seed, 8, 0, 0), v.data(), N);
    sample_gauss(Stream(seed, 9, 0, 0), e0.data(), N);
    sample_gauss(Stream(seed, 10, 0, 0), e1.data(), N);
    parallel_for(level, [&](int i) {
        const u64 t = ctx->mod[i];
        u64 *c0 = h_ct_out + ((size_t)0 * level + i) * N;
        u64 *c1 = h_ct_out + ((size_t)1 * level + i) * N;
        const u64 *b = h_pk + ((size_t)0 * L + i) * N;
        const u64 *a = h_pk + ((size_t)1 * L + i) * N;
        std::vector<u64> vh(N);
        small_to_ntt(ctx, i, v.data(), vh.data());
        for (u64 x = 0; x < N; x++) c0[x] = signed_residue(h_coeffs[x] + (int64_t)e0[x], t);
        ntt(ctx, i, c0);
        small_to_ntt(ctx, i, e1.data(), c1);
        for (u64 x = 0; x < N; x++) {
            const u64 w0 = c0[x] + mul_mod(vh[x], b[x], t), w1 = c1[x] + mul_mod(vh[x], a[x], t);
            c0[x] = w0 >= t ? w0 - t : w0;
            c1[x] = w1 >= t ? w1 - t : w1;
        }
    });
    return HE_OK;
}

// unsigned 192-bit helper for the CRT of up to three limbs
struct U192 {
    u64 w[3];
};
static U192 u192_from(u128 v) { return U192{{(u64)v, (u64)(v >> 64), 0}}; }
static U192 u192_mul64(U192 a, u64 b)
{
    U192 r;
    u128 c = 0;
    for (int i = 0; i < 3; i++) {
        c += (u128)a.w[i] * b;
        r.w[i] = (u64)c;
        c >>= 64;
    }
    return r;
}
static U192 u192_add(U192 a, U192 b)
{
    U192 r;
    u128 c = 0;
    for (int i = 0; i < 3; i++) {
        c += (u128)a.w[i] + b.w[i];
        r.w[i] = (u64)c;
        c >>= 64;
    }
    return r;
}
static U192 u192_sub(U192 a, U192 b)
{
    U192 r;
    int borrow = 0;
    for (int i = 0; i < 3; i++) {
        u128 d = (u128)a.w[i] - b.w[i] - borrow;
        r.w[i] = (u64)d;
        borrow = (d >> 64) ? 1 : 0;
    }
    return r;
}
static int u192_cmp(U192 a, U192 b)
{
    for (int i = 2; i >= 0; i--)
        if (a.w[i] != b.w[i]) return a.w[i] < b.w[i] ? -1 : 1;
    return 0;
}
static U192 u192_shr1(U192 a)
{
    U192 r;
    r.w[0] = (a.w[0] >> 1) | (a.w[1] << 63);
    r.w[1] = (a.w[1] >> 1) | (a.w[2] << 63);
    r.w[2] = a.w[2] >> 1;
    return r;
}
static double u192_to_double(U192 a)
{
    return std::ldexp((double)a.w[2], 128) + std::ldexp((double)a.w[1], 64) + (double)a.w[0];
}

extern "C" int32_t he_decrypt_coeffs(const he_ctx *ctx, const he_sk *sk, const uint64_t *h_ct, int32_t level,
                                     double *h_coeffs)
{
    if (!ctx || !sk || !h_ct || !h_coeffs || sk->ctx != ctx) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    const u64 N = ctx->N;
    const int nl = std::min(level, 3);
    std::vector<u64> res((size_t)nl * N);
    parallel_for(nl, [&](int i) {
        const u64 t = ctx->mod[i];
        const u64 *c0 = h_ct + ((size_t)0 * level + i) * N;
        const u64 *c1 = h_ct + ((size_t)1 * level + i) * N;
        const u64 *s = sk->s_ntt.data() + (size_t)i * N;
        u64 *o = res.data() + (size_t)i * N;
        for (u64 x = 0; x < N; x++) {
            u64 v = c0[x] + mul_mod(c1[x], s[x], t);
            o[x] = v >= t ? v - t : v;
        }
        intt(ctx, i, o);
    });
    // mixed-radix reconstruction: v = a0 + a1 q0 + a2 q0 q1, then the centred representative
    const u64 q0 = ctx->mod[0], q1 = nl > 1 ? ctx->mod[1] : 1, q2 = nl > 2 ? ctx->mod[2] : 1;
    const u64 inv01 = nl > 1 ? inv_mod(q0 % q1, q1) : 0;
    const u64 inv012 = nl > 2 ? inv_mod(mul_mod(q0 % q2, q1 % q2, q2), q2) : 0;
    U192 Q = u192_from((u128)q0);
    if (nl > 1) Q = u192_mul64(Q, q1);
    if (nl > 2) Q = u192_mul64(Q, q2);
    const U192 half = u192_shr1(Q);
    for (u64 x = 0; x < N; x++) {
        const u64 a0 = res[x];
        U192 v = u192_from((u128)a0);
        if (nl > 1) {
            const u64 r1 = res[N + x];
            const u64 a1 = mul_mod((r1 + q1 - a0 % q1) % q1, inv01, q1);
            u128 low = (u128)a0 + (u128)a1 * q0; // < q0 q1
            v = u192_from(low);
            if (nl > 2) {
                const u64 r2 = res[2 * N + x];
                const u64 low2 = (u64)(low % q2);
                const u64 a2 = mul_mod((r2 + q2 - low2) % q2, inv012, q2);
                U192 hi = u192_mul64(u192_mul64(u192_from((u128)a2), q0), q1);
                v = u192_add(v, hi);
            }
        }
        h_coeffs[x] = u192_cmp(v, half) > 0 ? -u192_to_double(u192_sub(Q, v)) : u192_to_double(v);
    }
    return HE_OK;
}

extern "C" int32_t he_decrypt(const he_ctx *ctx, const he_sk *sk, const uint64_t *h_ct, int32_t level, double scale,
                              double *h_re, double *h_im)
{
    if (!ctx) return HE_EINVAL;
    std::vector<double> m(ctx->N);
    int32_t rc = he_decrypt_coeffs(ctx, sk, h_ct, level, m.data());
    if (rc != HE_OK) return rc;
    return he_decode(ctx, m.data(), scale, h_re, h_im);
}
