// Internal structures of the RNS-CKKS library: host tables, their device images, handles.
#pragma once
#include <cstdint>
#include <functional>
#include <string>
#include <vector>

#include "he.h"

typedef uint64_t u64;
typedef unsigned __int128 u128;

// A constant w together with floor(w * 2^64 / q): lets the device compute w*x mod q with one
// high product and two low products (Shoup's method).
struct alignas(16) ShoupConst {
    u64 w;
    u64 wp;
};

// Per-modulus scalars the kernels need.
struct ModConst {
    u64 q;
    u64 one_p;    // floor(2^64 / q): reduces any 64-bit word to [0, 2q)
    ShoupConst r; // 2^64 mod q: folds the high word of a 128-bit sum
    double qd;    // q as a double when q < 2^50 (the FP64 arithmetic applies), else 0
    double qinvd; // 1/q rounded to nearest
};

// Device image of all tables.  Pointers are device pointers.
struct DevTables {
    const ModConst *mod;       // [M]
    const ShoupConst *tw_fwd;  // [M][N]  psi^brv(i)
    const ShoupConst *tw_inv;  // [M][N]  psi^-brv(i)
    const ShoupConst *ninv;    // [M][2]  N^-1 and psi^-brv(1) * N^-1 (last inverse stage)
    // the same three tables as balanced residues in (-q/2, q/2) stored as doubles (moduli < 2^50)
    const double *twd_fwd;     // [M][N]
    const double *twd_inv;     // [M][N]
    const double *ninvd;       // [M][2]
    // ModUp constants for digit j holding a active limbs (1 <= a <= alpha), slot (j*alpha + a-1):
    const ShoupConst *up_inv;  // [dnum*alpha][alpha]      (D/q_i)^-1 mod q_i
    const u64 *up_hat;         // [dnum*alpha][alpha][M]   (D/q_i) mod t
    const u64 *up_hat_p;       // the same shape: floor(((D/q_i) mod t) 2^64 / t), for products on the integer path
    const double *up_inv_d;    // balanced doubles of the same (0 where the modulus is >= 2^50)
    const double *up_hat_d;
    const double *up_hat_dh;   // (D/q_i) 2^31 mod t, for sources split at bit 31
    int up_split;              // some ciphertext prime is >= 2^50: FP64 targets split their sources
    // corrected conversions: 1.0 / (double)modulus for every modulus, and D mod t for the digit slots of up_hat
    const double *rq;          // [M]
    const u64 *up_dmod;        // [dnum*alpha][M]
    const double *up_dmod_d;   // balanced doubles of the same (0 where the modulus is >= 2^50)
    // ModDown constants
    const ShoupConst *dn_inv;  // [K]      (P/p_k)^-1 mod p_k
    const u64 *dn_hat;         // [K][L]   (P/p_k) mod q_i
    const ShoupConst *dn_pinv; // [L]      P^-1 mod q_i
    const double *dn_inv_d;    // [K]
    const double *dn_hat_d;    // [K][L]
    const double *dn_hat_dh;   // [K][L]   (P/p_k) 2^31 mod q_i
    const double *dn_pinv_d;   // [L]
    const u64 *dn_pmod;        // [L]      P mod q_i
    const double *dn_pmod_d;   // [L]
    int dn_split;              // some special prime is >= 2^50
    // ModDown from such primes onto a modulus q below 2^50 with 2^50 mod q small (|.| < 2^40, as for primes just
    // below a power of two): a source y = yh 2^50 + yl is first folded to yh (2^50 mod q) + yl, exact in a double
    const double *dn_r50_d;    // [L]  2^50 mod q_i, balanced
    int dn_fold;               // every floating-point ciphertext modulus qualifies
    // Rescale: q_l^-1 mod q_i
    const ShoupConst *rs_inv;  // [L][L]
    const double *rs_inv_d;    // [L][L]
    // ModDown and rescale in one step: (P q_l)^-1 mod q_i
    const ShoupConst *rsp_inv; // [L][L]
    const double *rsp_inv_d;   // [L][L]
};

struct ProfRecord {
    int kid;
    double bytes;
    void *a, *b; // hipEvent_t pair
};

struct he_ctx {
    int logN = 0, L = 0, K = 0, dnum = 0, alpha = 0, M = 0;
    u64 N = 0;
    int device = -1;
    std::vector<u64> mod;            // [M]
    std::vector<u64> psi;            // [M]
    std::vector<ModConst> modc;      // [M]
    std::vector<ShoupConst> tw_fwd;  // [M][N]
    std::vector<ShoupConst> tw_inv;  // [M][N]
    std::vector<ShoupConst> ninv;    // [M][2]
    std::vector<double> twd_fwd, twd_inv, ninvd;
    std::vector<ShoupConst> up_inv;
    std::vector<u64> up_hat;
    std::vector<double> up_inv_d, up_hat_d, up_hat_dh, dn_inv_d, dn_hat_d, dn_hat_dh, dn_pinv_d, dn_pmod_d, rs_inv_d, rsp_inv_d;
    std::vector<u64> dn_pmod;
    std::vector<double> rq, up_dmod_d, dn_r50_d;
    bool dn_fold = false;
    std::vector<u64> up_dmod, up_hat_p;
    int exact_conv = 0; // corrected base conversions selected (he_ctx_set_conversion)
    bool up_split = false, dn_split = false;
    std::vector<ShoupConst> dn_inv;
    std::vector<u64> dn_hat;
    std::vector<ShoupConst> dn_pinv;
    std::vector<ShoupConst> rs_inv, rsp_inv;
    // encode/decode tables
    std::vector<double> root_re, root_im; // exp(i pi e / N), e < 2N
    std::vector<uint32_t> slot_exp;       // 5^j mod 2N
    DevTables dev{};
    std::vector<void *> dev_allocs;
    u64 *static_scratch = nullptr; // address, on this context's device, of the library's file-scope scratch array
    mutable std::string hip_err;
    bool prof_on = false;
    std::vector<ProfRecord> prof;
};

struct he_sk {
    const he_ctx *ctx = nullptr;
    std::vector<int8_t> s;      // coefficients
    std::vector<u64> s_ntt;     // [M][N]
};

struct he_evk {
    const he_ctx *ctx = nullptr;
    u64 galois = 1;             // 1 = relinearisation key
    std::vector<u64> host;      // [dnum][2][M][N] (kept when the context has no device)
    u64 *dev = nullptr;         // device copy
};

// ---- host arithmetic (host_math.cpp) ------------------------------------------------------------
namespace hostmath {
u64 mul_mod(u64 a, u64 b, u64 q);
u64 pow_mod(u64 b, u64 e, u64 q);
u64 inv_mod(u64 a, u64 q);
ShoupConst shoup(u64 w, u64 q);
u64 least_primitive_root(u64 q);
unsigned bit_reverse(unsigned x, int bits);
// in-place negacyclic NTT / inverse on one limb with the context's tables
void ntt(const he_ctx *c, int mi, u64 *a);
void intt(const he_ctx *c, int mi, u64 *a);
void parallel_for(int n, const std::function<void(int)> &f);
} // namespace hostmath

// ---- device launchers (kernels.hip) ---------------------------------------------------------------
int32_t dev_upload_tables(he_ctx *c);
void dev_free_tables(he_ctx *c);
int32_t dev_upload_evk(he_evk *k);
void dev_free_evk(he_evk *k);
