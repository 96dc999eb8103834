// Device-side entry points of the RNS-CKKS library: table upload, kernel launch sequences of
// NTT, Mult (tensor product + relinearisation), Rotate (hybrid key switching), rescale and
// rotate-and-sum.  The kernels are in kernels_ntt.h, kernels_ks.h and kernels_elem.h.
//
// Key switch of a polynomial d (NTT domain, `level` limbs) with key evk, Galois element g:
//   1. inverse NTT of d, its column pass also multiplying limb i by (D/q_i)^-1      -> y  (ws.x)
//   2. forward NTT of every raised limb (digit j, modulus t outside the digit), the
//      column pass summing y_i (D/q_i mod t) on the fly (ModUp)                     -> raised
//   3. inner product with the key, reading the digits through the index map of g
//      and the digit's own limbs straight from d                                     -> u
//   4. inverse NTT of the special limbs of u, scaled by (P/p_k)^-1                   (in place)
//   5. forward NTT of the 2*level ModDown corrections, column pass summing
//      y_k (P/p_k mod q_i) over centred digits y_k, block pass finishing out = (u - ntt) P^-1 + addend       -> out
// Hoisted rotations share steps 1-2.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <functional>
#include <mutex>
#include <vector>

#include "kernels_elem.h"
#include "launch.h"

#define HIP_TRY(ctx, expr)                                                                                           \
    do {                                                                                                             \
        hipError_t e_ = (expr);                                                                                      \
        if (e_ != hipSuccess) {                                                                                      \
            (ctx)->hip_err = std::string(#expr) + ": " + hipGetErrorString(e_);                                      \
            return HE_EHIP;                                                                                          \
        }                                                                                                            \
    } while (0)

// Scratch array of he_hrot_noalloc: the workspace of one rotation for callers that cannot allocate and pass
// none.  Every GPU the library runs on holds its own copy at its own address; in host code the name below is
// only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned long long scratch[HE_STATIC_SCRATCH_BYTES / sizeof(unsigned long long)];

// Address of `scratch` on the context's device, asked for once per device (the caller has made that device
// current) and kept: kernels and copies take this pointer, never the array's name.
static int32_t static_scratch_address(he_ctx *c)
{
    static std::mutex mu;
    static u64 *per_device[64] = {};
    std::lock_guard<std::mutex> lock(mu);
    if (c->device < 0 || c->device >= 64) return HE_EINVAL;
    if (!per_device[c->device]) {
        void *p = nullptr;
        HIP_TRY(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) {
            c->hip_err = "hipGetSymbolAddress(scratch) returned a null address";
            return HE_EHIP;
        }
        per_device[c->device] = (u64 *)p;
    }
    c->static_scratch = per_device[c->device];
    return HE_OK;
}

template <class Tv> static int32_t upload(he_ctx *c, const std::vector<Tv> &v, const Tv **out)
{
    void *p = nullptr;
    const size_t bytes = std::max<size_t>(v.size() * sizeof(Tv), 16);
    HIP_TRY(c, hipMalloc(&p, bytes));
    c->dev_allocs.push_back(p);
    if (!v.empty()) HIP_TRY(c, hipMemcpy(p, v.data(), v.size() * sizeof(Tv), hipMemcpyHostToDevice));
    *out = (const Tv *)p;
    return HE_OK;
}

int32_t dev_upload_tables(he_ctx *c)
{
    if (c->logN != 12 && c->logN != 16 && c->logN != 17) return HE_EINVAL;
    if (c->alpha > 8 || c->K > 8 || c->M > 64) return HE_EINVAL; // conversion kernels are built for up to 8 sources
    if (c->logN == 17 && (c->alpha > 4 || c->K > 4)) return HE_EINVAL; // ... and for up to 4 at N = 2^17
    HIP_TRY(c, hipSetDevice(c->device));
    int32_t rc;
    if ((rc = static_scratch_address(c)) != HE_OK) return rc; // once per context, with its device current
#define UP(field)                                                                                                    \
    if ((rc = upload(c, c->field, &c->dev.field)) != HE_OK) return rc;
    if ((rc = upload(c, c->modc, &c->dev.mod)) != HE_OK) return rc;
    UP(tw_fwd) UP(tw_inv) UP(ninv) UP(twd_fwd) UP(twd_inv) UP(ninvd)
    UP(up_inv) UP(up_hat) UP(up_inv_d) UP(up_hat_d) UP(up_hat_dh) UP(rq) UP(up_dmod) UP(up_dmod_d) UP(up_hat_p) UP(dn_r50_d)
    UP(dn_inv) UP(dn_hat) UP(dn_pinv) UP(dn_inv_d) UP(dn_hat_d) UP(dn_hat_dh) UP(dn_pinv_d) UP(dn_pmod) UP(dn_pmod_d)
    UP(rs_inv) UP(rs_inv_d) UP(rsp_inv) UP(rsp_inv_d)
#undef UP
    c->dev.up_split = c->up_split ? 1 : 0;
    c->dev.dn_split = c->dn_split ? 1 : 0;
    c->dev.dn_fold = c->dn_fold ? 1 : 0;
    return HE_OK;
}

void dev_free_tables(he_ctx *c)
{
    for (void *p : c->dev_allocs) (void)hipFree(p);
    c->dev_allocs.clear();
}

// Device form of a key: limbs of a modulus below 2^50 (the floating-point path) hold balanced residues as
// doubles (v, or v - q above (q-1)/2), the other limbs the residues themselves.  The inner product then
// multiplies key words without converting them, and products with |word| <= q/2 are exact for wider inputs.
int32_t dev_upload_evk(he_evk *k)
{
    he_ctx *c = const_cast<he_ctx *>(k->ctx);
    const size_t N = c->N, limbs = (size_t)c->dnum * 2 * c->M;
    std::vector<u64> img;
    try {
        img.resize(limbs * N);
    } catch (...) {
        return HE_ENOMEM;
    }
    std::atomic<bool> bad(false);
    hostmath::parallel_for((int)limbs, [&](int l) {
        const ModConst &m = c->modc[l % c->M];
        const u64 *src = k->host.data() + (size_t)l * N, half = (m.q - 1) / 2;
        u64 *dst = img.data() + (size_t)l * N;
        bool b = false;
        for (size_t n = 0; n < N; n++) {
            const u64 v = src[n];
            b |= v >= m.q;
            if (m.qd != 0.0) {
                const double d = v > half ? -(double)(m.q - v) : (double)v;
                memcpy(&dst[n], &d, sizeof(d));
            } else
                dst[n] = v;
        }
        if (b) bad = true;
    });
    if (bad) return HE_EINVAL; // a residue that is not below its modulus
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, hipMalloc((void **)&k->dev, img.size() * sizeof(u64)));
    hipError_t e = hipMemcpy(k->dev, img.data(), img.size() * sizeof(u64), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        c->hip_err = std::string("hipMemcpy (key upload): ") + hipGetErrorString(e);
        (void)hipFree(k->dev);
        k->dev = nullptr;
        return HE_EHIP;
    }
    return HE_OK;
}

void dev_free_evk(he_evk *k)
{
    if (k->dev) (void)hipFree(k->dev);
    k->dev = nullptr;
}

extern "C" int32_t he_evk_to_host(const he_evk *evk, uint64_t *h_out)
{
    if (!evk || !h_out) return HE_EINVAL;
    const he_ctx *c = evk->ctx;
    const size_t N = c->N, limbs = (size_t)c->dnum * 2 * c->M, words = limbs * N;
    if (!evk->dev) {
        memcpy(h_out, evk->host.data(), words * sizeof(u64));
        return HE_OK;
    }
    he_ctx *cm = const_cast<he_ctx *>(c);
    HIP_TRY(cm, hipMemcpy(h_out, evk->dev, words * sizeof(u64), hipMemcpyDeviceToHost));
    hostmath::parallel_for((int)limbs, [&](int l) { // back from the device form to residues
        const ModConst &m = c->modc[l % c->M];
        if (m.qd == 0.0) return;
        u64 *w = h_out + (size_t)l * N;
        for (size_t n = 0; n < N; n++) {
            double d;
            memcpy(&d, &w[n], sizeof(d));
            w[n] = d < 0.0 ? m.q - (u64)(-d) : (u64)d;
        }
    });
    return HE_OK;
}

// ---- optional per-kernel timing with HIP events on the launch stream (he_profile_start/stop)
static const char *const kKernelNames[KID_COUNT] = {
    "k_ntt_fwd_cols", "k_ntt_fwd_cols_modup", "k_ntt_fwd_cols_moddown", "k_ntt_fwd_cols_rescale", "k_ntt_fwd_cols_moddown_rescale",
    "k_ntt_fwd_blocks",
    "k_ntt_fwd_blocks_fin", "k_ntt_inv_blocks", "k_ntt_inv_cols", "k_limbwise", "k_cmult", "k_tensor", "k_inner_blocks"};

bool prof_events(he_ctx *c, int kid, double bytes, ProfRecord &r)
{
    r.kid = kid;
    r.bytes = bytes;
    r.a = r.b = nullptr;
    if (hipEventCreate((hipEvent_t *)&r.a) != hipSuccess) return false;
    if (hipEventCreate((hipEvent_t *)&r.b) != hipSuccess) {
        (void)hipEventDestroy((hipEvent_t)r.a);
        return false;
    }
    c->prof.push_back(r);
    return true;
}

// launchers of the context's ring size (dev_upload_tables has checked that it is one of the three)
static const DevLaunch &dev_launch(const he_ctx *c)
{
    static const DevLaunch tables[3] = {
        [] { DevLaunch t{}; dev_launch_n12(t); return t; }(),
        [] {
            DevLaunch t{};
            dev_launch_cols16_0(t), dev_launch_cols16_1(t), dev_launch_cols16_2(t), dev_launch_cols16_3(t);
            dev_launch_cols16_4(t), dev_launch_cols16_5(t), dev_launch_n16_blocks(t);
            dev_launch_cols_ex16_1(t), dev_launch_cols_ex16_2(t), dev_launch_cols_ex16_4(t);
            return t;
        }(),
        [] {
            DevLaunch t{};
            dev_launch_cols17_0(t), dev_launch_cols17_1(t), dev_launch_cols17_2(t), dev_launch_cols17_3(t);
            dev_launch_cols17_4(t), dev_launch_cols17_5(t), dev_launch_n17_blocks(t);
            dev_launch_cols_ex17_1(t), dev_launch_cols_ex17_2(t), dev_launch_cols_ex17_4(t);
            return t;
        }(),
    };
    return tables[c->logN == 12 ? 0 : c->logN == 16 ? 1 : 2];
}

extern "C" int32_t he_profile_start(he_ctx *ctx)
{
    if (!ctx) return HE_EINVAL;
    if (ctx->device < 0) return HE_ENODEV;
    ctx->prof_on = true;
    return HE_OK;
}

extern "C" int32_t he_profile_stop(he_ctx *ctx, he_kernel_stat *out, int32_t max_out, int32_t *n_out)
{
    if (!ctx || !out || !n_out || max_out < 0) return HE_EINVAL;
    ctx->prof_on = false;
    double ms[KID_COUNT] = {0}, bytes[KID_COUNT] = {0};
    int64_t cnt[KID_COUNT] = {0};
    int32_t rc = HE_OK;
    for (ProfRecord &r : ctx->prof) {
        float t = 0.f;
        if (r.a && r.b && hipEventSynchronize((hipEvent_t)r.b) == hipSuccess &&
            hipEventElapsedTime(&t, (hipEvent_t)r.a, (hipEvent_t)r.b) == hipSuccess) {
            ms[r.kid] += t;
            bytes[r.kid] += r.bytes;
            cnt[r.kid]++;
        } else
            rc = HE_EHIP;
        if (r.a) (void)hipEventDestroy((hipEvent_t)r.a);
        if (r.b) (void)hipEventDestroy((hipEvent_t)r.b);
    }
    ctx->prof.clear();
    int32_t n = 0;
    for (int k = 0; k < KID_COUNT; k++) {
        if (!cnt[k]) continue;
        if (n < max_out) {
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, kKernelNames[k], sizeof(out[n].name) - 1);
            out[n].launches = cnt[k];
            out[n].total_ms = ms[k];
            out[n].bytes = bytes[k];
        }
        n++;
    }
    *n_out = n;
    if (n > max_out && rc == HE_OK) rc = HE_EINVAL; // the caller's array is too small: n_out says how many are needed
    return rc;
}

static inline int32_t launch_ok(he_ctx *c)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        c->hip_err = std::string("kernel launch: ") + hipGetErrorString(e);
        return HE_EHIP;
    }
    return HE_OK;
}

// ---- limb lists -----------------------------------------------------------------------------------

struct LimbList {
    std::vector<int> slot, src, mod;
    void add(int s, int m) { slot.push_back(s), src.push_back(s), mod.push_back(m); }
    void add(int s, int from, int m) { slot.push_back(s), src.push_back(from), mod.push_back(m); }
    int size() const { return (int)slot.size(); }
};

// calls launch(batch, count) for chunks of at most HE_MAXB limbs; within a chunk the limbs on the integer path
// (moduli of 2^50 and above) take about three times longer and are scheduled first, so that the others fill in
// behind them
template <class F> static int32_t for_batches(he_ctx *c, const LimbList &l, F launch)
{
    const int total = l.size();
    std::vector<int> order(HE_MAXB);
    // chunks of equal size (even, so that pairs of limbs stay together) rather than full ones and a small rest
    const int nchunks = (total + HE_MAXB - 1) / HE_MAXB;
    const int per = nchunks ? std::min(HE_MAXB, ((total + nchunks - 1) / nchunks + 1) & ~1) : 0;
    for (int off = 0; off < total; off += per) {
        const int nb = std::min(per, total - off);
        for (int b = 0; b < nb; b++) order[b] = off + b;
        std::stable_partition(order.begin(), order.begin() + nb, [&](int b) { return c->modc[l.mod[b]].qd == 0.0; });
        LimbBatch lb;
        for (int b = 0; b < nb; b++) {
            const int o = order[b];
            lb.slot[b] = (uint16_t)l.slot[o];
            lb.src[b] = (uint16_t)l.src[o];
            lb.mod[b] = (uint8_t)l.mod[o];
        }
        launch(lb, nb);
        int32_t rc = launch_ok(c);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

static ConvArgs conv_args(const he_ctx *c, const u64 *src, int level, int dst_stride = 1 << 30, int src_stride = 0)
{
    ConvArgs cv;
    cv.src = src;
    cv.level = level;
    cv.L = c->L;
    cv.K = c->K;
    cv.alpha = c->alpha;
    cv.dst_stride = dst_stride;
    cv.src_stride = src_stride;
    cv.src2 = nullptr;
    cv.src2_stride = 0;
    cv.rs_mod = level - 1;
    cv.rs_nl = level - 1;
    cv.exact = c->exact_conv;
    memset(cv.op_level, 0, sizeof(cv.op_level));
    return cv;
}

static FinArgs fin_args(const u64 *u, u64 *out, const u64 *add, const ShoupConst *cst, const double *cst_d, int u_cstride,
                        int nl, int mode, unsigned g, int dst_stride, int u_stride, int out_stride, int add_stride)
{
    FinArgs fa;
    fa.u = u, fa.out = out, fa.add = add, fa.self = nullptr;
    fa.cst = cst, fa.cst_d = cst_d, fa.cst2 = nullptr, fa.cst2_d = nullptr;
    fa.u_cstride = u_cstride, fa.out_cstride = nl, fa.add_cstride = nl, fa.self_stride = 0, fa.nl = nl, fa.mode = mode;
    fa.g = g;
    fa.hoisted = 0;
    fa.dst_stride = dst_stride, fa.u_stride = u_stride, fa.out_stride = out_stride, fa.add_stride = add_stride;
    return fa;
}
static const HoistOuts kNoHoistOuts = {};
static const HoistKeys kNoHoistKeys = {};
static const FinArgs kNoFin = fin_args(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 1, 0, 1u, 1 << 30, 0, 0, 0);

// Forward NTT of the listed limbs of `data`.  pro selects what the column pass transforms (the
// limb's own content, or a base conversion of cv.src); with fin != nullptr the block pass writes
// (u - ntt) * const + addend to fin->out instead of the transform itself.
// src_limbs = number of source limbs the prologue reads in total (for the byte count).
// int_blocks_only: the block pass runs only for limbs on the integer path (the others are finished by the
// kernel that consumes them).
static int32_t ntt_forward(he_ctx *c, hipStream_t st, u64 *data, const LimbList &l, int pro, const ConvArgs &cv,
                           const FinArgs *fin, int src_limbs, bool int_blocks_only = false,
                           const HoistOuts *hoist = nullptr)
{
    const HoistOuts &ho = hoist ? *hoist : kNoHoistOuts;
    const bool wide = std::max(c->alpha, c->K) > 4;
    const double N8 = (double)c->N * 8.0;
    const DevLaunch &dl = dev_launch(c);
    int32_t rc = for_batches(c, l, [&](const LimbBatch &lb, int nb) {
        const double cols_bytes = pro == PRO_LOAD ? 2.0 * nb * N8 : (double)(src_limbs + nb) * N8;
        const int kid_cols = pro == PRO_LOAD      ? KID_FWD_COLS
                             : pro == PRO_MODUP   ? KID_FWD_COLS_MODUP
                             : pro == PRO_MODDOWN ? KID_FWD_COLS_MODDOWN
                             : pro == PRO_MODDOWN_RS ? KID_FWD_COLS_MODDOWN_RS
                                                  : KID_FWD_COLS_RESCALE;
        (cv.exact && dl.fwd_cols_ex[pro] ? dl.fwd_cols_ex[pro] : dl.fwd_cols[pro])(c, st, kid_cols, cols_bytes, wide, data, lb, nb, cv);
        if (fin) {
            // reads the transform's input, the minuend and the addend, writes the result
            const double b = (double)nb * N8 * (3.0 + (fin->mode == 1 || fin->mode == 3 ? 1.0 : fin->mode == 2 ? 0.5 : fin->mode == 4 ? 1.5 : 0.0));
            dl.fwd_blocks(c, st, b, true, data, lb, nb, *fin, ho);
        } else if (!int_blocks_only)
            dl.fwd_blocks(c, st, 2.0 * nb * N8, false, data, lb, nb, kNoFin, kNoHoistOuts);
    });
    if (rc != HE_OK || !int_blocks_only) return rc;
    // block pass of the integer-path limbs alone, after all column passes: few launches, each as large as possible
    LimbList li;
    for (int b = 0; b < l.size(); b++)
        if (c->modc[l.mod[b]].qd == 0.0) li.add(l.slot[b], l.src[b], l.mod[b]);
    return for_batches(c, li, [&](const LimbBatch &lb, int nb) {
        dl.fwd_blocks(c, st, 2.0 * nb * N8, false, data, lb, nb, kNoFin, kNoHoistOuts);
    });
}

// Inverse NTT: limb b read at src + l.src[b]*N, result at dst + l.slot[b]*N; scale folds a base
// conversion constant into the final 1/N.
// blocks_done: the block pass has already been applied (by the inner-product kernel), in place in dst.
static int32_t ntt_inverse(he_ctx *c, hipStream_t st, const u64 *src, u64 *dst, const LimbList &l, int scale,
                           const ConvArgs &cv, bool blocks_done = false)
{
    const double N8 = (double)c->N * 8.0;
    const DevLaunch &dl = dev_launch(c);
    return for_batches(c, l, [&](const LimbBatch &lb, int nb) {
        const double bytes = 2.0 * nb * N8;
        if (!blocks_done) dl.inv_blocks(c, st, bytes, src, dst, lb, nb);
        dl.inv_cols(c, st, bytes, scale, dst, lb, nb, cv);
    });
}

static int32_t dev_guard(he_ctx *c)
{
    if (!c) return HE_EINVAL;
    if (c->device < 0) return HE_ENODEV;
    return HE_OK;
}

static int32_t ntt_api(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream, bool inv)
{
    int32_t rc = dev_guard(ctx);
    if (rc != HE_OK) return rc;
    if (!d_limbs || !h_mod_idx || batch < 0) return HE_EINVAL;
    for (int b = 0; b < batch; b++)
        if (h_mod_idx[b] < 0 || h_mod_idx[b] >= ctx->M) return HE_EINVAL;
    const ConvArgs cv = conv_args(ctx, nullptr, 1);
    // limb slots are 16-bit: walk the buffer in windows
    const int WIN = 32768;
    for (int off = 0; off < batch; off += WIN) {
        const int nb = std::min(WIN, batch - off);
        LimbList l;
        for (int b = 0; b < nb; b++) l.add(b, h_mod_idx[off + b]);
        u64 *base = d_limbs + (size_t)off * ctx->N;
        rc = inv ? ntt_inverse(ctx, (hipStream_t)stream, base, base, l, SCALE_NONE, cv)
                 : ntt_forward(ctx, (hipStream_t)stream, base, l, PRO_LOAD, cv, nullptr, 0);
        if (rc != HE_OK) return rc;
    }
    return HE_OK;
}

extern "C" int32_t he_ntt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream)
{
    return ntt_api(ctx, d_limbs, h_mod_idx, batch, stream, false);
}
extern "C" int32_t he_intt(he_ctx *ctx, uint64_t *d_limbs, const int32_t *h_mod_idx, int32_t batch, void *stream)
{
    return ntt_api(ctx, d_limbs, h_mod_idx, batch, stream, true);
}

static int32_t level_guard(he_ctx *c, int level)
{
    int32_t rc = dev_guard(c);
    if (rc != HE_OK) return rc;
    if (level < 1 || level > c->L) return HE_ELEVEL;
    return HE_OK;
}

// a, b, out: [count] operations of `limbs` limbs each, strides sa / sb / so limbs between operations
static int32_t limbwise(he_ctx *c, const u64 *a, const u64 *b, u64 *out, int level, int op, int limbs, int b_limbs,
                        void *stream, int count = 1, int sa = 0, int sb = 0, int so = 0)
{
    int32_t rc = level_guard(c, level);
    if (rc != HE_OK) return rc;
    if (!a || !b || !out || count < 1 || limbs > 65535 || count > 65535) return HE_EINVAL;
    dim3 grid((unsigned)(c->N / 256), (unsigned)limbs, (unsigned)count);
    KLAUNCH(c, (hipStream_t)stream, KID_LIMBWISE, (double)count * (2 * limbs + b_limbs) * c->N * 8.0, (k_limbwise), grid, a,
            b, out, c->dev, op, level, b_limbs, c->logN, sa, sb, so);
    return launch_ok(c);
}

static bool count_ok(int level, int count) { return count >= 1 && (long)count * 2 * level <= 65535; }

extern "C" int32_t he_add_batch(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                                int32_t count, void *stream)
{
    if (!count_ok(level, count)) return HE_EINVAL;
    return limbwise(ctx, d_a, d_b, d_out, level, 0, count * 2 * level, count * 2 * level, stream);
}
extern "C" int32_t he_sub_batch(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                                int32_t count, void *stream)
{
    if (!count_ok(level, count)) return HE_EINVAL;
    return limbwise(ctx, d_a, d_b, d_out, level, 1, count * 2 * level, count * 2 * level, stream);
}
extern "C" int32_t he_pmult_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *d_pt, uint64_t *d_out,
                                  int32_t level, int32_t count, void *stream)
{
    if (!count_ok(level, count)) return HE_EINVAL;
    return limbwise(ctx, d_ct, d_pt, d_out, level, 2, count * 2 * level, level, stream);
}
extern "C" int32_t he_add(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                          void *stream)
{
    return he_add_batch(ctx, d_a, d_b, d_out, level, 1, stream);
}
extern "C" int32_t he_sub(he_ctx *ctx, const uint64_t *d_a, const uint64_t *d_b, uint64_t *d_out, int32_t level,
                          void *stream)
{
    return he_sub_batch(ctx, d_a, d_b, d_out, level, 1, stream);
}
extern "C" int32_t he_pmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *d_pt, uint64_t *d_out, int32_t level,
                            void *stream)
{
    return he_pmult_batch(ctx, d_ct, d_pt, d_out, level, 1, stream);
}

extern "C" int32_t he_pmult_sum(he_ctx *ctx, const uint64_t *const *h_d_cts, const uint64_t *const *h_d_pts,
                                int32_t count, uint64_t *d_out, int32_t level, void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!h_d_cts || !h_d_pts || !d_out || count < 1 || count > PMULT_SUM_MAX) return HE_EINVAL;
    PmultSumArgs a;
    memset(&a, 0, sizeof(a));
    for (int k = 0; k < count; k++) {
        if (!h_d_cts[k] || !h_d_pts[k]) return HE_EINVAL;
        a.ct[k] = h_d_cts[k];
        a.pt[k] = h_d_pts[k];
    }
    a.count = count;
    dim3 grid((unsigned)(ctx->N / 256), (unsigned)(2 * level));
    KLAUNCH(ctx, (hipStream_t)stream, KID_LIMBWISE, (double)(3 * count + 2) * level * ctx->N * 8.0, (k_pmult_sum), grid, a,
            d_out, ctx->dev, level, ctx->logN);
    return launch_ok(ctx);
}

static int32_t scalar_args(he_ctx *ctx, const uint64_t *h_scalar, int level, bool with_companion, ScalarArgs &sc)
{
    memset(&sc, 0, sizeof(sc));
    for (int i = 0; i < level; i++) {
        if (h_scalar[i] >= ctx->mod[i]) return HE_EINVAL;
        if (with_companion)
            sc.s[i] = hostmath::shoup(h_scalar[i], ctx->mod[i]);
        else
            sc.s[i].w = h_scalar[i];
    }
    return HE_OK;
}

extern "C" int32_t he_cmult_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out,
                                  int32_t level, int32_t count, void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!d_ct || !h_scalar || !d_out || !count_ok(level, count)) return HE_EINVAL;
    ScalarArgs sc;
    if ((rc = scalar_args(ctx, h_scalar, level, true, sc)) != HE_OK) return rc;
    dim3 grid((unsigned)(ctx->N / 256), (unsigned)(count * 2 * level));
    KLAUNCH(ctx, (hipStream_t)stream, KID_CMULT, 4.0 * count * level * ctx->N * 8.0, (k_cmult), grid, d_ct, d_out, ctx->dev,
            sc, level, ctx->logN);
    return launch_ok(ctx);
}
extern "C" int32_t he_cmult(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out, int32_t level,
                            void *stream)
{
    return he_cmult_batch(ctx, d_ct, h_scalar, d_out, level, 1, stream);
}

extern "C" int32_t he_add_const_batch(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out,
                                      int32_t level, int32_t count, void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!d_ct || !h_scalar || !d_out || !count_ok(level, count)) return HE_EINVAL;
    ScalarArgs sc;
    if ((rc = scalar_args(ctx, h_scalar, level, false, sc)) != HE_OK) return rc;
    dim3 grid((unsigned)(ctx->N / 256), (unsigned)(count * 2 * level));
    KLAUNCH(ctx, (hipStream_t)stream, KID_LIMBWISE, 4.0 * count * level * ctx->N * 8.0, (k_addconst), grid, d_ct, d_out,
            ctx->dev, sc, level, ctx->logN);
    return launch_ok(ctx);
}
extern "C" int32_t he_add_const(he_ctx *ctx, const uint64_t *d_ct, const uint64_t *h_scalar, uint64_t *d_out,
                                int32_t level, void *stream)
{
    return he_add_const_batch(ctx, d_ct, h_scalar, d_out, level, 1, stream);
}

extern "C" int32_t he_moddrop_batch(he_ctx *ctx, const uint64_t *d_ct, int32_t in_level, uint64_t *d_out,
                                    int32_t out_level, int32_t count, void *stream)
{
    int32_t rc = level_guard(ctx, in_level);
    if (rc != HE_OK) return rc;
    if (out_level < 1 || out_level > in_level) return HE_ELEVEL;
    if (!d_ct || !d_out || d_ct == d_out || count < 1) return HE_EINVAL;
    const size_t N = ctx->N;
    // one row per (operation, component): the first out_level limbs of in_level
    hipError_t e = hipMemcpy2DAsync(d_out, (size_t)out_level * N * sizeof(u64), d_ct, (size_t)in_level * N * sizeof(u64),
                                    (size_t)out_level * N * sizeof(u64), (size_t)count * 2, hipMemcpyDeviceToDevice,
                                    (hipStream_t)stream);
    if (e != hipSuccess) {
        ctx->hip_err = std::string("hipMemcpy2DAsync: ") + hipGetErrorString(e);
        return HE_EHIP;
    }
    return HE_OK;
}
extern "C" int32_t he_moddrop(he_ctx *ctx, const uint64_t *d_ct, int32_t in_level, uint64_t *d_out, int32_t out_level,
                              void *stream)
{
    return he_moddrop_batch(ctx, d_ct, in_level, d_out, out_level, 1, stream);
}

// the key-switch kernels read and write 16-byte pairs
static inline bool misaligned16(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// ---- workspace layout (in limbs of N words), per operation of a batch
struct WsLayout {
    size_t x, d, raised, u, r, tmp, total;
};
static WsLayout ws_layout(const he_ctx *c, int level)
{
    const size_t Ma = level + c->K, beta = (level + c->alpha - 1) / c->alpha;
    WsLayout w;
    size_t o = 0;
    w.x = o, o += std::max(level, 2); // y: inverse transform of the switched polynomial, scaled
    w.d = o, o += level;              // d2 of the tensor product (NTT domain)
    w.raised = o, o += beta * Ma;     // raised digits (slots of a digit's own limbs stay unused)
    w.u = o, o += 2 * Ma;             // inner products
    w.r = o, o += 2 * level;          // ModDown / rescale corrections
    w.tmp = o, o += 2 * level;        // rotate_sum: the rotated ciphertext
    w.total = o;
    return w;
}

extern "C" int32_t he_workspace_bytes(const he_ctx *ctx, int32_t level, int32_t count, size_t *out)
{
    if (!ctx || !out || count < 1) return HE_EINVAL;
    if (level < 1 || level > ctx->L) return HE_ELEVEL;
    *out = ws_layout(ctx, level).total * (size_t)count * ctx->N * sizeof(u64);
    return HE_OK;
}

// limb slots are 16-bit offsets from a buffer's base
static bool batch_fits(const WsLayout &w, int count) { return count >= 1 && w.total * (size_t)count <= 65535; }

// Steps 1-2 of the key switch for `count` polynomials: operation o reads its NTT-domain input at
// d_ntt + o*d_stride limbs and works in ws + o*w.total limbs.  Raised limbs on the floating-point path
// are left as the column pass wrote them (the inner-product kernel finishes them).
static int32_t ks_raise(he_ctx *c, const u64 *d_ntt, int d_stride, u64 *ws, const WsLayout &w, int level, int count,
                        hipStream_t st)
{
    const size_t N = c->N;
    const int K = c->K, Ma = level + K, beta = (level + c->alpha - 1) / c->alpha, W = (int)w.total;
    LimbList l;
    for (int o = 0; o < count; o++)
        for (int i = 0; i < level; i++) l.add(o * W + i, o * d_stride + i, i);
    const ConvArgs cv = conv_args(c, ws + w.x * N, level, W, W);
    int32_t rc = ntt_inverse(c, st, d_ntt, ws + w.x * N, l, SCALE_MODUP, cv);
    if (rc != HE_OK) return rc;
    LimbList r;
    for (int o = 0; o < count; o++)
        for (int j = 0; j < beta; j++) {
            const int lo = j * c->alpha, hi = std::min(lo + c->alpha, level);
            for (int a = 0; a < Ma; a++) {
                if (a >= lo && a < hi) continue;
                r.add(o * W + j * Ma + a, a < level ? a : c->L + (a - level));
            }
        }
    return ntt_forward(c, st, ws + w.raised * N, r, PRO_MODUP, cv, nullptr, level * count, true);
}

// Step 3 and the inverse transform of step 4: u and, in its special limbs, the scaled coefficient-domain digits.
// hoist != nullptr: `count` rotations of one raised input (operation 0's workspace), operation o with key hoist->evk[o].
// shared_raised = false: per-operation keys as well, but every operation has its own raised input.
static int32_t ks_inner(he_ctx *c, const he_evk *evk, const u64 *d_ntt, int d_stride, u64 *ws, const WsLayout &w,
                        int level, int count, hipStream_t st, const HoistKeys *hoist = nullptr, bool shared_raised = true)
{
    const size_t N = c->N;
    const int K = c->K, Ma = level + K, beta = (level + c->alpha - 1) / c->alpha, W = (int)w.total;
    const unsigned g = (unsigned)evk->galois;
    if (misaligned16(ws) || misaligned16(d_ntt) || misaligned16(evk->dev)) return HE_EINVAL; // entry points check first
    dim3 grid(inner_grid((unsigned)(N / INNER_TILE), (unsigned)Ma, (unsigned)count));
    InnerArgs ia;
    ia.raised = ws + w.raised * N, ia.d = d_ntt, ia.evk = evk->dev, ia.u = ws + w.u * N;
    ia.level = level, ia.L = c->L, ia.K = K, ia.alpha = c->alpha, ia.beta = beta;
    ia.g = g, ia.raised_stride = hoist && shared_raised ? 0 : W, ia.u_stride = W, ia.d_stride = d_stride, ia.inv_special = 1;
    ia.hoisted = hoist ? 1 : 0, ia.count = count;
    const HoistKeys &hk = hoist ? *hoist : kNoHoistKeys;
    // Bytes by the definition of the step, each operand once per launch: every operation writes 2 limbs per active
    // modulus; beta digits per active modulus are read once per raised input (one for hoisted rotations, else one
    // per operation); 2 beta key limbs per active modulus are read once per distinct key of the launch.
    int keys = 1;
    if (hoist) {
        std::vector<const u64 *> seen(hoist->evk, hoist->evk + count);
        std::sort(seen.begin(), seen.end());
        keys = (int)(std::unique(seen.begin(), seen.end()) - seen.begin());
    }
    const int inputs = hoist && shared_raised ? 1 : count;
    const double inner_bytes = ((double)inputs * beta + 2.0 * count + 2.0 * beta * keys) * Ma * N * 8.0;
    dev_launch(c).inner(c, st, inner_bytes, grid.x, ia, hk);
    int32_t rc = launch_ok(c);
    if (rc != HE_OK) return rc;
    LimbList sp;
    for (int o = 0; o < count; o++)
        for (int cc = 0; cc < 2; cc++)
            for (int k = 0; k < K; k++) sp.add(o * W + cc * Ma + level + k, c->L + k);
    const ConvArgs cv = conv_args(c, ws + w.u * N, level, W, W);
    return ntt_inverse(c, st, ws + w.u * N, ws + w.u * N, sp, SCALE_MODDOWN, cv, true);
}

// Steps 3-5.  Operation o writes out + o*out_stride limbs; mode / c0 (+ o*c0_stride): the addend of
// the final step (see FinArgs).
static int32_t ks_apply(he_ctx *c, const he_evk *evk, const u64 *d_ntt, int d_stride, u64 *ws, const WsLayout &w,
                        int level, int count, u64 *out, int out_stride, const u64 *c0, int c0_stride, int mode,
                        hipStream_t st)
{
    const size_t N = c->N;
    const int Ma = level + c->K, W = (int)w.total;
    int32_t rc = ks_inner(c, evk, d_ntt, d_stride, ws, w, level, count, st);
    if (rc != HE_OK) return rc;
    const ConvArgs cv = conv_args(c, ws + w.u * N, level, W, W);
    LimbList r;
    for (int o = 0; o < count; o++)
        for (int cc = 0; cc < 2; cc++)
            for (int i = 0; i < level; i++) r.add(o * W + cc * level + i, i);
    FinArgs fa = fin_args(ws + w.u * N, out, c0, c->dev.dn_pinv, c->dev.dn_pinv_d, Ma, level, mode,
                          (unsigned)evk->galois, W, W, out_stride, c0_stride);
    if (mode == 4) fa.self = c0, fa.self_stride = c0_stride; // c0 points at the whole input ciphertext [2][level][N]
    return ntt_forward(c, st, ws + w.r * N, r, PRO_MODDOWN, cv, &fa, 2 * c->K * count);
}

static int32_t ks_guard(he_ctx *c, const he_evk *evk, int level, int count, void *ws, size_t ws_bytes)
{
    int32_t rc = level_guard(c, level);
    if (rc != HE_OK) return rc;
    if (!evk || evk->ctx != c || !evk->dev) return HE_ENOKEY;
    if (!ws || misaligned16(ws) || misaligned16(evk->dev)) return HE_EINVAL;
    const WsLayout w = ws_layout(c, level);
    if (!batch_fits(w, count)) return HE_EINVAL;
    if (ws_bytes < w.total * (size_t)count * c->N * sizeof(u64)) return HE_EWORKSPACE;
    return HE_OK;
}

extern "C" int32_t he_hmult_relin_batch(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                                        uint64_t *d_out, int32_t level, int32_t count, void *d_ws, size_t ws_bytes,
                                        void *stream)
{
    int32_t rc = ks_guard(ctx, relin, level, count, d_ws, ws_bytes);
    if (rc != HE_OK) return rc;
    if (relin->galois != 1) return HE_ENOKEY;
    if (!d_a || !d_b || !d_out || misaligned16(d_a) || misaligned16(d_b) || misaligned16(d_out)) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const size_t N = ctx->N;
    const int W = (int)w.total;
    dim3 grid((unsigned)(N / 256), (unsigned)level, (unsigned)count);
    KLAUNCH(ctx, st, KID_TENSOR, 7.0 * count * level * N * 8.0, (k_tensor), grid, d_a, d_b, d_out, ws + w.d * N, ctx->dev,
            level, ctx->logN, W, 2 * level);
    if ((rc = launch_ok(ctx)) != HE_OK) return rc;
    if ((rc = ks_raise(ctx, ws + w.d * N, W, ws, w, level, count, st)) != HE_OK) return rc;
    return ks_apply(ctx, relin, ws + w.d * N, W, ws, w, level, count, d_out, 2 * level, nullptr, 0, 1, st);
}

extern "C" int32_t he_hmult_relin(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                                  uint64_t *d_out, int32_t level, void *d_ws, size_t ws_bytes, void *stream)
{
    return he_hmult_relin_batch(ctx, relin, d_a, d_b, d_out, level, 1, d_ws, ws_bytes, stream);
}

// Mult followed by rescale with one forward transform per output limb.  After the inner product: ModDown of
// the last limb alone (c_last = (u - ntt(r)) P^-1 + d), its inverse transform t, then for every other limb
// the column pass transforms r + P t_centred and the block pass finishes (u - ntt) (P q_l)^-1 + d q_l^-1.
extern "C" int32_t he_hmult_relin_rescale_batch(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a,
                                                const uint64_t *d_b, uint64_t *d_out, int32_t level, int32_t count,
                                                void *d_ws, size_t ws_bytes, void *stream)
{
    int32_t rc = ks_guard(ctx, relin, level, count, d_ws, ws_bytes);
    if (rc != HE_OK) return rc;
    if (relin->galois != 1) return HE_ENOKEY;
    if (level < 2) return HE_ELEVEL;
    if (!d_a || !d_b || !d_out || misaligned16(d_a) || misaligned16(d_b) || misaligned16(d_out)) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const size_t N = ctx->N;
    const int W = (int)w.total, K = ctx->K, Ma = level + K, L = ctx->L;
    u64 *d01 = ws + w.tmp * N; // per operation [2][level][N]: d0, d1 of the tensor product
    dim3 grid((unsigned)(N / 256), (unsigned)level, (unsigned)count);
    KLAUNCH(ctx, st, KID_TENSOR, 7.0 * count * level * N * 8.0, (k_tensor), grid, d_a, d_b, d01, ws + w.d * N, ctx->dev,
            level, ctx->logN, W, W);
    if ((rc = launch_ok(ctx)) != HE_OK) return rc;
    if ((rc = ks_raise(ctx, ws + w.d * N, W, ws, w, level, count, st)) != HE_OK) return rc;
    if ((rc = ks_inner(ctx, relin, ws + w.d * N, W, ws, w, level, count, st)) != HE_OK) return rc;
    u64 *rbuf = ws + w.r * N;
    ConvArgs cv = conv_args(ctx, ws + w.u * N, level, W, W);
    cv.src2 = rbuf;
    cv.src2_stride = W;
    // ModDown of the last limb of both components, in place in the correction buffer
    LimbList last;
    for (int o = 0; o < count; o++)
        for (int cc = 0; cc < 2; cc++) last.add(o * W + cc * level + level - 1, level - 1);
    FinArgs fl = fin_args(ws + w.u * N, rbuf, d01, ctx->dev.dn_pinv, ctx->dev.dn_pinv_d, Ma, level, 3, 1u, W, W, W, W);
    if ((rc = ntt_forward(ctx, st, rbuf, last, PRO_MODDOWN, cv, &fl, 2 * K * count)) != HE_OK) return rc;
    if ((rc = ntt_inverse(ctx, st, rbuf, rbuf, last, SCALE_NONE, cv)) != HE_OK) return rc;
    // every other limb: ModDown and rescale corrections in one transform
    LimbList rest;
    for (int o = 0; o < count; o++)
        for (int cc = 0; cc < 2; cc++)
            for (int i = 0; i < level - 1; i++) rest.add(o * W + cc * level + i, i);
    FinArgs fa = fin_args(ws + w.u * N, d_out, d01, ctx->dev.rsp_inv + (size_t)(level - 1) * L,
                          ctx->dev.rsp_inv_d + (size_t)(level - 1) * L, Ma, level, 3, 1u, W, W, 2 * (level - 1), W);
    fa.out_cstride = level - 1;
    fa.cst2 = ctx->dev.rs_inv + (size_t)(level - 1) * L;
    fa.cst2_d = ctx->dev.rs_inv_d + (size_t)(level - 1) * L;
    return ntt_forward(ctx, st, rbuf, rest, PRO_MODDOWN_RS, cv, &fa, (2 * K + 2) * count);
}

extern "C" int32_t he_hmult_relin_rescale(he_ctx *ctx, const he_evk *relin, const uint64_t *d_a, const uint64_t *d_b,
                                          uint64_t *d_out, int32_t level, void *d_ws, size_t ws_bytes, void *stream)
{
    return he_hmult_relin_rescale_batch(ctx, relin, d_a, d_b, d_out, level, 1, d_ws, ws_bytes, stream);
}

extern "C" int32_t he_hrot_many(he_ctx *ctx, const he_evk *const *rots, int32_t count, const uint64_t *d_ct,
                                uint64_t *const *h_d_outs, int32_t level, void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || count < 1 || !h_d_outs) return HE_EINVAL;
    int32_t rc;
    for (int r = 0; r < count; r++) {
        if ((rc = ks_guard(ctx, rots[r], level, 1, d_ws, ws_bytes)) != HE_OK) return rc;
        if (rots[r]->galois == 1) return HE_ENOKEY;
        if (!h_d_outs[r] || h_d_outs[r] == d_ct || misaligned16(h_d_outs[r])) return HE_EINVAL;
    }
    if (!d_ct || misaligned16(d_ct)) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const u64 *c1 = d_ct + (size_t)level * ctx->N;
    if ((rc = ks_raise(ctx, c1, 0, ws, w, level, 1, st)) != HE_OK) return rc;
    const size_t N = ctx->N;
    const int W = (int)w.total, Ma = level + ctx->K;
    // With workspace for several operations the rotations share every launch: operation o keeps its inner
    // products and ModDown corrections in workspace o, all read the raised digits of workspace 0.
    const int fit = (int)std::min<size_t>(ws_bytes / (w.total * N * sizeof(u64)), HOIST_MAX);
    int r = 0;
    while (fit >= 2 && count - r >= 2 && batch_fits(w, std::min(fit, count - r))) {
        const int nb = std::min(fit, count - r);
        HoistKeys hk = {};
        HoistOuts ho = {};
        for (int o = 0; o < nb; o++) {
            hk.evk[o] = rots[r + o]->dev;
            hk.g[o] = ho.g[o] = (unsigned)rots[r + o]->galois;
            ho.out[o] = h_d_outs[r + o];
        }
        if ((rc = ks_inner(ctx, rots[r], c1, 0, ws, w, level, nb, st, &hk)) != HE_OK) return rc;
        const ConvArgs cv = conv_args(ctx, ws + w.u * N, level, W, W);
        LimbList lr;
        for (int o = 0; o < nb; o++)
            for (int cc = 0; cc < 2; cc++)
                for (int i = 0; i < level; i++) lr.add(o * W + cc * level + i, i);
        FinArgs fa = fin_args(ws + w.u * N, nullptr, d_ct, ctx->dev.dn_pinv, ctx->dev.dn_pinv_d, Ma, level, 2, 1u, W, W, 0, 0);
        fa.hoisted = 1;
        if ((rc = ntt_forward(ctx, st, ws + w.r * N, lr, PRO_MODDOWN, cv, &fa, 2 * ctx->K * nb, false, &ho)) != HE_OK)
            return rc;
        r += nb;
    }
    for (; r < count; r++)
        if ((rc = ks_apply(ctx, rots[r], c1, 0, ws, w, level, 1, h_d_outs[r], 0, d_ct, 0, 2, st)) != HE_OK) return rc;
    return HE_OK;
}

// in: operation o at d_ct + o*in_stride limbs; out: operation o at d_out + o*out_stride limbs.
// plus_input: the result is ct + Rotate(ct) instead of Rotate(ct).
static int32_t hrot_batch_to(he_ctx *ctx, const he_evk *rot, const u64 *d_ct, int in_stride, u64 *d_out, int out_stride,
                             int level, int count, void *d_ws, size_t ws_bytes, hipStream_t st, bool plus_input = false)
{
    int32_t rc = ks_guard(ctx, rot, level, count, d_ws, ws_bytes);
    if (rc != HE_OK) return rc;
    if (rot->galois == 1) return HE_ENOKEY;
    if (!d_ct || !d_out || d_ct == d_out || misaligned16(d_ct) || misaligned16(d_out)) return HE_EINVAL;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const u64 *c1 = d_ct + (size_t)level * ctx->N;
    if ((rc = ks_raise(ctx, c1, in_stride, ws, w, level, count, st)) != HE_OK) return rc;
    return ks_apply(ctx, rot, c1, in_stride, ws, w, level, count, d_out, out_stride, d_ct, in_stride, plus_input ? 4 : 2, st);
}

extern "C" int32_t he_hrot_batch(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                                 int32_t count, void *d_ws, size_t ws_bytes, void *stream)
{
    return hrot_batch_to(ctx, rot, d_ct, 2 * level, d_out, 2 * level, level, count, d_ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int32_t he_hrot(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                           void *d_ws, size_t ws_bytes, void *stream)
{
    return he_hrot_batch(ctx, rot, d_ct, d_out, level, 1, d_ws, ws_bytes, stream);
}

// he_hrot on the library's own scratch array: no workspace argument, no allocation.
extern "C" int32_t he_hrot_noalloc(he_ctx *ctx, const he_evk *rot, const uint64_t *d_ct, uint64_t *d_out, int32_t level,
                                   void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!ctx->static_scratch) return HE_EHIP;
    if (ws_layout(ctx, level).total * ctx->N * sizeof(u64) > HE_STATIC_SCRATCH_BYTES) return HE_ESCRATCH;
    return hrot_batch_to(ctx, rot, d_ct, 2 * level, d_out, 2 * level, level, 1, ctx->static_scratch, HE_STATIC_SCRATCH_BYTES,
                         (hipStream_t)stream);
}

extern "C" int32_t he_hrot_batch_keys(he_ctx *ctx, const he_evk *const *rots, const uint64_t *d_ct, uint64_t *d_out,
                                      int32_t level, int32_t count, void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || count < 1) return HE_EINVAL;
    int32_t rc;
    for (int r = 0; r < count; r++) {
        if ((rc = ks_guard(ctx, rots[r], level, 1, d_ws, ws_bytes)) != HE_OK) return rc;
        if (rots[r]->galois == 1) return HE_ENOKEY;
    }
    if (!d_ct || !d_out || d_ct == d_out || misaligned16(d_ct) || misaligned16(d_out)) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const WsLayout w = ws_layout(ctx, level);
    const size_t N = ctx->N;
    const int W = (int)w.total, Ma = level + ctx->K, ct_limbs = 2 * level;
    int fit = (int)std::min<size_t>(ws_bytes / (w.total * N * sizeof(u64)), HOIST_MAX);
    while (fit > 1 && !batch_fits(w, fit)) fit--;
    for (int r = 0; r < count;) {
        const int nb = std::min(fit, count - r);
        const u64 *in = d_ct + (size_t)r * ct_limbs * N, *c1 = in + (size_t)level * N;
        if ((rc = ks_raise(ctx, c1, ct_limbs, ws, w, level, nb, st)) != HE_OK) return rc;
        HoistKeys hk = {};
        HoistOuts ho = {};
        for (int o = 0; o < nb; o++) {
            hk.evk[o] = rots[r + o]->dev;
            hk.g[o] = ho.g[o] = (unsigned)rots[r + o]->galois;
            ho.out[o] = d_out + (size_t)(r + o) * ct_limbs * N;
        }
        if ((rc = ks_inner(ctx, rots[r], c1, ct_limbs, ws, w, level, nb, st, &hk, false)) != HE_OK) return rc;
        const ConvArgs cv = conv_args(ctx, ws + w.u * N, level, W, W);
        LimbList lr;
        for (int o = 0; o < nb; o++)
            for (int cc = 0; cc < 2; cc++)
                for (int i = 0; i < level; i++) lr.add(o * W + cc * level + i, i);
        FinArgs fa = fin_args(ws + w.u * N, nullptr, in, ctx->dev.dn_pinv, ctx->dev.dn_pinv_d, Ma, level, 2, 1u, W, W, 0, ct_limbs);
        fa.hoisted = 1;
        if ((rc = ntt_forward(ctx, st, ws + w.r * N, lr, PRO_MODDOWN, cv, &fa, 2 * ctx->K * nb, false, &ho)) != HE_OK)
            return rc;
        r += nb;
    }
    return HE_OK;
}

// Rotations at mixed levels in shared launches.  The buffers of every operation are laid out for the largest
// level of its group (workspace stride, limbs per raised digit and per component), an operation below that
// level simply has no limbs between its own level and the layout's, and fewer digits.
extern "C" int32_t he_hrot_batch_levels(he_ctx *ctx, const he_evk *const *rots, const int32_t *h_levels, const uint64_t *d_ct,
                                        uint64_t *d_out, int32_t count, void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || !h_levels || count < 1) return HE_EINVAL;
    int32_t rc;
    int lmax_all = 0;
    for (int r = 0; r < count; r++) {
        if ((rc = level_guard(ctx, h_levels[r])) != HE_OK) return rc;
        lmax_all = std::max(lmax_all, (int)h_levels[r]);
    }
    for (int r = 0; r < count; r++) {
        if ((rc = ks_guard(ctx, rots[r], lmax_all, 1, d_ws, ws_bytes)) != HE_OK) return rc;
        if (rots[r]->galois == 1) return HE_ENOKEY;
    }
    if (!d_ct || !d_out || d_ct == d_out || misaligned16(d_ct) || misaligned16(d_out)) return HE_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const size_t N = ctx->N;
    const int K = ctx->K, alpha = ctx->alpha, L = ctx->L;
    size_t done_limbs = 0; // limbs of the operations already processed (inputs and outputs are packed alike)
    for (int r = 0; r < count;) {
        // group: as many operations as the workspace holds at the layout of their largest level
        int nb = 0, lmax = 0;
        while (r + nb < count && nb < HOIST_MAX) {
            const int lm = std::max(lmax, (int)h_levels[r + nb]);
            const WsLayout wl = ws_layout(ctx, lm);
            if (!batch_fits(wl, nb + 1) || wl.total * (size_t)(nb + 1) * N * sizeof(u64) > ws_bytes) break;
            lmax = lm, nb++;
        }
        if (nb == 0) return HE_EWORKSPACE;
        const WsLayout w = ws_layout(ctx, lmax);
        const int W = (int)w.total, Ma = lmax + K;
        const u64 *in0 = d_ct + done_limbs * N;
        u64 *out0 = d_out + done_limbs * N;
        std::vector<size_t> off(nb + 1, 0); // limb offset of operation o within the group
        for (int o = 0; o < nb; o++) off[o + 1] = off[o] + 2 * (size_t)h_levels[r + o];
        if (off[nb] > 65535) return HE_EINVAL;
        ConvArgs cv = conv_args(ctx, ws + w.x * N, lmax, W, W);
        HoistKeys hk = {};
        HoistOuts ho = {};
        for (int o = 0; o < nb; o++) {
            const int lo = h_levels[r + o];
            cv.op_level[o] = hk.level[o] = ho.cstride[o] = (uint8_t)lo;
            hk.evk[o] = rots[r + o]->dev;
            hk.g[o] = ho.g[o] = (unsigned)rots[r + o]->galois;
            hk.d[o] = in0 + (off[o] + lo) * N; // c1
            ho.add[o] = in0 + off[o] * N;      // c0
            ho.out[o] = out0 + off[o] * N;
        }
        // 1. inverse transform of every c1 limb, scaled for its digit's conversion
        LimbList l;
        for (int o = 0; o < nb; o++)
            for (int i = 0; i < h_levels[r + o]; i++) l.add(o * W + i, (int)(off[o] + h_levels[r + o] + i), i);
        if ((rc = ntt_inverse(ctx, st, in0, ws + w.x * N, l, SCALE_MODUP, cv)) != HE_OK) return rc;
        // 2. raised digits
        LimbList rl;
        int src_limbs = 0;
        for (int o = 0; o < nb; o++) {
            const int lo = h_levels[r + o], beta = (lo + alpha - 1) / alpha;
            src_limbs += lo;
            for (int j = 0; j < beta; j++) {
                const int dlo = j * alpha, dhi = std::min(dlo + alpha, lo);
                for (int a = 0; a < Ma; a++) {
                    if ((a >= dlo && a < dhi) || (a >= lo && a < lmax)) continue;
                    rl.add(o * W + j * Ma + a, a < lmax ? a : L + (a - lmax));
                }
            }
        }
        if ((rc = ntt_forward(ctx, st, ws + w.raised * N, rl, PRO_MODUP, cv, nullptr, src_limbs, true)) != HE_OK) return rc;
        // 3. inner products (block pass of the special limbs' inverse transform included) and 4. its column pass
        if (misaligned16(ws)) return HE_EINVAL;
        InnerArgs ia;
        ia.raised = ws + w.raised * N, ia.d = in0, ia.evk = rots[r]->dev, ia.u = ws + w.u * N;
        ia.level = lmax, ia.L = L, ia.K = K, ia.alpha = alpha, ia.beta = (lmax + alpha - 1) / alpha;
        ia.g = 1u, ia.raised_stride = W, ia.u_stride = W, ia.d_stride = 0, ia.inv_special = 1, ia.hoisted = 1, ia.count = nb;
        // bytes by definition: digits and results per operation, each distinct key once at the largest level it serves
        double inner_bytes = 0.0;
        std::vector<std::pair<const u64 *, int>> key_level;
        for (int o = 0; o < nb; o++) {
            const int lo = h_levels[r + o], beta = (lo + alpha - 1) / alpha;
            inner_bytes += (double)(beta + 2) * (lo + K) * N * 8.0;
            bool found = false;
            for (auto &kl : key_level)
                if (kl.first == hk.evk[o]) kl.second = std::max(kl.second, lo), found = true;
            if (!found) key_level.push_back({hk.evk[o], lo});
        }
        for (const auto &kl : key_level) inner_bytes += 2.0 * ((kl.second + alpha - 1) / alpha) * (kl.second + K) * N * 8.0;
        dev_launch(ctx).inner(ctx, st, inner_bytes, inner_grid((unsigned)(N / INNER_TILE), (unsigned)Ma, (unsigned)nb), ia, hk);
        if ((rc = launch_ok(ctx)) != HE_OK) return rc;
        LimbList sp;
        for (int o = 0; o < nb; o++)
            for (int cc = 0; cc < 2; cc++)
                for (int k = 0; k < K; k++) sp.add(o * W + cc * Ma + lmax + k, L + k);
        const ConvArgs cu = conv_args(ctx, ws + w.u * N, lmax, W, W);
        if ((rc = ntt_inverse(ctx, st, ws + w.u * N, ws + w.u * N, sp, SCALE_MODDOWN, cu, true)) != HE_OK) return rc;
        // 5. ModDown: corrections transformed and applied, plus the rotated c0
        LimbList lr;
        for (int o = 0; o < nb; o++)
            for (int cc = 0; cc < 2; cc++)
                for (int i = 0; i < h_levels[r + o]; i++) lr.add(o * W + cc * lmax + i, i);
        FinArgs fa = fin_args(ws + w.u * N, nullptr, in0, ctx->dev.dn_pinv, ctx->dev.dn_pinv_d, Ma, lmax, 2, 1u, W, W, 0, 0);
        fa.hoisted = 1;
        if ((rc = ntt_forward(ctx, st, ws + w.r * N, lr, PRO_MODDOWN, cu, &fa, 2 * K * nb, false, &ho)) != HE_OK) return rc;
        done_limbs += off[nb];
        r += nb;
    }
    return HE_OK;
}

extern "C" int32_t he_rotate_sum_batch(he_ctx *ctx, const he_evk *const *rots, int32_t n_rot, uint64_t *d_ct,
                                       int32_t level, int32_t count, void *d_ws, size_t ws_bytes, void *stream)
{
    if (!rots || n_rot < 0) return HE_EINVAL;
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (!d_ws || !d_ct) return HE_EINVAL;
    const WsLayout w = ws_layout(ctx, level);
    if (!batch_fits(w, count)) return HE_EINVAL;
    if (ws_bytes < w.total * (size_t)count * ctx->N * sizeof(u64)) return HE_EWORKSPACE;
    if (misaligned16(d_ct)) return HE_EINVAL;
    for (int k = 0; k < n_rot; k++) { // every key is checked before the first launch
        if ((rc = ks_guard(ctx, rots[k], level, count, d_ws, ws_bytes)) != HE_OK) return rc;
        if (rots[k]->galois == 1) return HE_ENOKEY;
    }
    // ct + Rotate(ct) is written by the key switch itself, alternately into the workspace (operation o at
    // tmp + o*w.total limbs) and back into d_ct
    u64 *tmp = (u64 *)d_ws + w.tmp * ctx->N;
    const int W = (int)w.total;
    hipStream_t st = (hipStream_t)stream;
    bool in_tmp = false;
    for (int k = 0; k < n_rot; k++) {
        rc = in_tmp ? hrot_batch_to(ctx, rots[k], tmp, W, d_ct, 2 * level, level, count, d_ws, ws_bytes, st, true)
                    : hrot_batch_to(ctx, rots[k], d_ct, 2 * level, tmp, W, level, count, d_ws, ws_bytes, st, true);
        if (rc != HE_OK) return rc;
        in_tmp = !in_tmp;
    }
    if (in_tmp) {
        const size_t row = (size_t)2 * level * ctx->N * sizeof(u64);
        hipError_t e = hipMemcpy2DAsync(d_ct, row, tmp, (size_t)W * ctx->N * sizeof(u64), row, (size_t)count,
                                        hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) {
            ctx->hip_err = std::string("hipMemcpy2DAsync: ") + hipGetErrorString(e);
            return HE_EHIP;
        }
    }
    return HE_OK;
}

extern "C" int32_t he_rotate_sum(he_ctx *ctx, const he_evk *const *rots, int32_t count, uint64_t *d_ct, int32_t level,
                                 void *d_ws, size_t ws_bytes, void *stream)
{
    return he_rotate_sum_batch(ctx, rots, count, d_ct, level, 1, d_ws, ws_bytes, stream);
}

extern "C" int32_t he_rescale_batch(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level, int32_t count,
                                    void *d_ws, size_t ws_bytes, void *stream)
{
    int32_t rc = level_guard(ctx, level);
    if (rc != HE_OK) return rc;
    if (level < 2) return HE_ELEVEL;
    if (!d_ct || !d_out || !d_ws || d_ct == d_out) return HE_EINVAL;
    const WsLayout w = ws_layout(ctx, level);
    if (!batch_fits(w, count)) return HE_EINVAL;
    if (ws_bytes < w.total * (size_t)count * ctx->N * sizeof(u64)) return HE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const size_t N = ctx->N;
    const int W = (int)w.total;
    u64 *t = ws + w.x * N; // per operation two limbs: the dropped limb of each component, coefficient domain
    u64 *r = ws + w.r * N; // per operation [2][level-1][N]
    LimbList last;
    for (int o = 0; o < count; o++)
        for (int c = 0; c < 2; c++) last.add(o * W + c, o * 2 * level + c * level + level - 1, level - 1);
    const ConvArgs cv = conv_args(ctx, t, level, W, W);
    if ((rc = ntt_inverse(ctx, st, d_ct, t, last, SCALE_NONE, cv)) != HE_OK) return rc;
    LimbList l;
    for (int o = 0; o < count; o++)
        for (int c = 0; c < 2; c++)
            for (int i = 0; i < level - 1; i++) l.add(o * W + c * (level - 1) + i, i);
    const FinArgs fa = fin_args(d_ct, d_out, nullptr, ctx->dev.rs_inv + (size_t)(level - 1) * ctx->L,
                                ctx->dev.rs_inv_d + (size_t)(level - 1) * ctx->L, level, level - 1, 0, 1u, W, 2 * level,
                                2 * (level - 1), 0);
    return ntt_forward(ctx, st, r, l, PRO_RESCALE, cv, &fa, 2 * count);
}

// ModRaise, the first step of bootstrapping: the centred coefficients of a level-1 ciphertext reduced modulo
// every q_i, i < level_out.
extern "C" int32_t he_modraise(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level_out, void *d_ws,
                               size_t ws_bytes, void *stream)
{
    int32_t rc = level_guard(ctx, level_out);
    if (rc != HE_OK) return rc;
    if (level_out < 2) return HE_ELEVEL;
    if (!d_ct || !d_out || !d_ws || d_ct == d_out) return HE_EINVAL;
    const WsLayout w = ws_layout(ctx, level_out);
    if (ws_bytes < w.total * ctx->N * sizeof(u64)) return HE_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    u64 *ws = (u64 *)d_ws;
    const size_t N = ctx->N;
    u64 *t = ws + w.x * N; // two limbs: the coefficient-domain components
    LimbList in;
    in.add(0, 0, 0);
    in.add(1, 1, 0);
    ConvArgs cv = conv_args(ctx, t, level_out, 1 << 30, 0);
    cv.rs_mod = 0;
    cv.rs_nl = level_out;
    if ((rc = ntt_inverse(ctx, st, d_ct, t, in, SCALE_NONE, cv)) != HE_OK) return rc;
    LimbList l;
    for (int c = 0; c < 2; c++)
        for (int i = 1; i < level_out; i++) l.add(c * level_out + i, i);
    if ((rc = ntt_forward(ctx, st, d_out, l, PRO_RESCALE, cv, nullptr, 2)) != HE_OK) return rc;
    // limb 0 of both components is the input itself
    hipError_t e = hipMemcpy2DAsync(d_out, (size_t)level_out * N * sizeof(u64), d_ct, N * sizeof(u64), N * sizeof(u64), 2,
                                    hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) {
        ctx->hip_err = std::string("hipMemcpy2DAsync: ") + hipGetErrorString(e);
        return HE_EHIP;
    }
    return HE_OK;
}

extern "C" int32_t he_rescale(he_ctx *ctx, const uint64_t *d_ct, uint64_t *d_out, int32_t level, void *d_ws,
                              size_t ws_bytes, void *stream)
{
    return he_rescale_batch(ctx, d_ct, d_out, level, 1, d_ws, ws_bytes, stream);
}
