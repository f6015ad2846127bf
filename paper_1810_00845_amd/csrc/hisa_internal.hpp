// Internal declarations shared by the translation units of libhisa.
// Host orchestration lives in hisa_api.hip; every arithmetic step runs in the
// kernels declared here (launch wrappers take plain pointers and sizes).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <set>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/hisa.h"

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

// Per-prime constants, one entry per prime q_0..q_{L-1}, p_0..p_{K-1}, device resident.
struct PrimeConst {
    u64 q;
    u64 r1, r0;        // floor(2^128 / q)
    u64 n_inv, n_inv_sh; // N^-1 mod q and its Shoup companion
    u64 half;          // floor(q / 2)
};

// fp64 view of a prime below 2^50 (exact modular arithmetic in doubles)
struct FpPrime {
    double p, pinv, half;
};

// Device pointers to the per-prime tables, [prime][N] each.
struct NttTables {
    const PrimeConst* primes;
    const u64* tw;     // psi^bitrev(i)
    const u64* tw_sh;  // Shoup companions
    const u64* itw;    // psi^-bitrev(i)
    const u64* itw_sh;
    // fp64 path (all primes below 2^50, 12 <= log2 N <= 15), else fp_ok = 0 and the pointers are null
    int fp_ok;
    const FpPrime* fprimes;
    const double* ftw;  // psi^bitrev(i), centred
    const double* utw;  // utw[m + k] = psi^(-k N/m), k < m = 2^t: inverse decimation-in-time twiddles
    const double* vtw;  // psi^-j / N
};

// Which polynomials a batched NTT launch touches: polynomial p (0 <= p <
// n_polys) sits at base + (p / period) * batch_stride + (p % period) * N and
// is transformed modulo prime prime_of[p % period]; a negative entry skips it.
#define HISA_MAX_PERIOD 256
struct PolyMap {
    int32_t period;
    int16_t prime_of[HISA_MAX_PERIOD];
};

// Optional extras of an inverse transform.
struct InttExtra {
    const u64* in;          // read from here instead of data (same PolyMap addressing with in_batch_stride); may be null
    u64 in_batch_stride;
    u64 galois;             // != 0: input index i reads the element that sigma_g moves to i (NTT-form automorphism)
    const u64* post;        // per period entry: final factor replacing N^-1 (already multiplied by N^-1), may be null
    const u64* post_sh;
    int out_entry0;         // output polynomial of entry e sits at (e - out_entry0) * N within its batch slot
};

// One fast base conversion: source primes src[0..a), all primes as targets.
struct ConvTable {
    int a;
    int src[HISA_MAX_Q];
    u64* d_inv_hat;     // [a]   (D/c_i)^-1 mod c_i
    u64* d_inv_hat_sh;  // [a]
    u64* d_hat;         // [a][total]  (D/c_i) mod t
    u64* d_dmod;        // [total]     D mod t
    std::vector<u64> inv_hat; // host copy
    double* d_hat_f;    // [a][total]  (D/c_i) mod t as centred doubles (fp64 path), may be null
};

struct DevBlock {
    void* ptr;
    size_t bytes;
    int refs;
};

#define HISA_MAGIC_CT 0x43544631u
#define HISA_MAGIC_PT 0x50544631u

struct hisa_ct {
    uint32_t magic;
    DevBlock* blk;
    u64* data;  // [polys][limbs][N], NTT form
    uint32_t polys, limbs;
    double scale;
};

struct hisa_pt {
    uint32_t magic;
    DevBlock* blk;
    u64* data;  // [limbs][N], NTT form
    uint32_t limbs;
    double scale;
};

struct SwitchKey {
    DevBlock* blk;
    u64* data;  // [dnum][2][total][N]: b then a, NTT form
};

struct hisa_ctx {
    hisa_params prm;
    uint32_t log_n, N, L, K, alpha, dnum, total;
    hipStream_t stream;
    std::vector<u64> mod, psi;  // q_0..q_{L-1}, p_0..p_{K-1}
    std::vector<PrimeConst> pc;
    PrimeConst* d_primes;
    u64 *d_tw, *d_tw_sh, *d_itw, *d_itw_sh;
    NttTables tabs;
    u64* d_secret;  // [total][N], NTT form
    std::map<u64, SwitchKey> keys;  // 0: relinearisation, else Galois element
    struct Analysis* analysis = nullptr;   // non-null between hisa_analysis_begin and hisa_analysis_end
    uint32_t fused_rescale = 0;            // hisa_set_fused_rescale: layers divide by q_{l-1} P at once where they can
    uint32_t merge_doublings = 0;          // hisa_set_merge_doublings: rotate-and-add chains as sums of rotations (0, 2..4)
    std::map<u64, SwitchKey> aux;   // small derived device tables, built on first use
    std::map<std::pair<int, int>, ConvTable> modup_tabs;  // (digit, size)
    ConvTable* moddown_tab;
    u64* d_pinv;      // [L] P^-1 mod q_i
    u64* d_pinv_sh;
    u64* d_pmod;      // [L] P mod q_i
    double *d_cos, *d_sin;  // [2N] roots of unity exp(i*pi*t/N)
    FpPrime* d_fprimes;     // fp64 path tables (null when not applicable)
    double *d_ftw, *d_utw, *d_vtw, *d_pinv_f;
    u64* d_gauss_cdt = nullptr;            // [gauss_cdt_n] floor(2^63 P(|X| <= k)) of the error distribution
    int gauss_cdt_n = 0;
    std::vector<i64> sparse_secret;        // secret_kind = 1: the secret's coefficients, drawn on the host
    double* d_moddown_hat_pin = nullptr;   // [K][total] (P/p_m) * P^-1 mod q_i, centred: ModDown's conversion with the division folded in
    uint32_t* d_pow5;       // [N/2] 5^j mod 2N
    double* d_fp_scratch;   // fp64 path: one polynomial per resident workgroup of the conversion kernels
    int fp_scratch_polys;
    std::unordered_map<size_t, std::vector<void*>> pool;
    size_t pool_bytes;
    std::map<uintptr_t, size_t> live;   // blocks handed out by dev_alloc and not yet back in the pool: start -> bytes
    u64 enc_counter;
    int device = -1;              // the GPU the context lives on (current when it was made)
    void* noalloc_ws = nullptr;   // that GPU's copy of the library's static scratch array (hisa_rot_left_noalloc)
    std::string err;
};

// ---- host helpers shared by hisa_api.hip and layers.hip ----
int fail(hisa_ctx* ctx, int code, const char* fmt, ...);

#define HIP_TRY(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t e__ = (expr);                                                                  \
        if (e__ != hipSuccess)                                                                    \
            return fail(ctx, e__ == hipErrorOutOfMemory ? HISA_ERR_OOM : HISA_ERR_HIP, "%s: %s", #expr, \
                        hipGetErrorString(e__));                                                  \
    } while (0)

#define TRY(expr)                  \
    do {                           \
        int rc__ = (expr);         \
        if (rc__ != HISA_OK) return rc__; \
    } while (0)

DevBlock* dev_alloc(hisa_ctx* ctx, size_t bytes);   // from the context's pool; null (and last_error set) on failure
void dev_release(hisa_ctx* ctx, DevBlock* b);
// 8-byte words from p to the end of the live pool block that holds p; 0 when no live block does
u64 dev_words_behind(const hisa_ctx* ctx, const void* p);

struct Temp {  // pooled scratch buffer for the duration of one call
    hisa_ctx* ctx;
    DevBlock* blk;
    struct None {};    // no buffer: the caller brought memory of its own
    Temp(hisa_ctx* c, size_t bytes) : ctx(c), blk(dev_alloc(c, bytes)) {}
    Temp(hisa_ctx* c, None) : ctx(c), blk(nullptr) {}
    Temp(hisa_ctx* c, size_t bytes, bool wanted) : ctx(c), blk(wanted ? dev_alloc(c, bytes) : nullptr) {}
    ~Temp() { dev_release(ctx, blk); }
    bool ok() const { return blk != nullptr; }
    u64* u() const { return (u64*)blk->ptr; }
    template <class T> T* as() const { return (T*)blk->ptr; }
    Temp(const Temp&) = delete;
    Temp& operator=(const Temp&) = delete;
};

static inline bool valid_ct(const hisa_ct* c) { return c && c->magic == HISA_MAGIC_CT; }
static inline bool valid_pt(const hisa_pt* p) { return p && p->magic == HISA_MAGIC_PT; }
static inline size_t ct_words(const hisa_ctx* ctx, uint32_t polys, uint32_t limbs) { return (size_t)polys * limbs * ctx->N; }

// n ciphertext handles that are views of one allocation, [n][polys][limbs][N]
int alloc_ct_batch(hisa_ctx* ctx, size_t n, uint32_t polys, uint32_t limbs, double scale, hisa_ct** out);
int alloc_pt(hisa_ctx* ctx, uint32_t limbs, double scale, hisa_pt** out);

// A batch of equally shaped ciphertexts as one strided array.  When the handles are not evenly
// spaced views of one allocation they are first copied side by side (tmp then owns the copy).
struct BatchIn {
    const u64* base = nullptr;
    u64 stride = 0;
    DevBlock* tmp = nullptr;
};
int gather_batch(hisa_ctx* ctx, const hisa_ct* const* cts, size_t n, BatchIn* bi);
int check_batch_shape(hisa_ctx* ctx, const hisa_ct* const* cts, size_t n, uint32_t polys);
PolyMap identity_map(int limbs);
// pieces of the fused fp64 key switch for sums that are formed before the division by P (hisa_api.hip)
bool fused_key_switch_available(const hisa_ctx* ctx);
int rotation_accumulators_fp(hisa_ctx* ctx, const u64* cts, u64 ct_bs, size_t B, int l, const int32_t* steps, int n_steps,
                             u64* acc, bool fold_c0 = false);
// out[b] = plain[b] + sum_s rotLeft(rot[s * Bn + b], steps[s]) with one division by P per output: rot holds
// n_steps * Bn ciphertexts [2][l][N], ct_bs words apart, rotation-major; every step rotates (its key is present);
// plain ([Bn] ciphertexts, plain_bs apart) may be null; out [Bn][2][l][N].  shared_input: rot holds Bn ciphertexts and
// every term of output b rotates rot[b] (one decomposition per output).  Dry runs count and return.
// rescale: the sum's divScalar is taken together with its division by P (moddown_rescale_fp): out [Bn][2][l - 1][N].
int rotate_sum_fp(hisa_ctx* ctx, const u64* rot, u64 ct_bs, int n_steps, const int32_t* steps, size_t Bn, int l,
                  const u64* plain, u64 plain_bs, u64* out, bool shared_input = false, bool rescale = false);
// The division by P and the divScalar by q_{l-1} in one base conversion: acc [B][2][l + K][N] (overwritten: the addend
// [B][add_polys][l][N] is first folded in, times P) -> out [B][2][l - 1][N] = (acc + P add) / (q_{l-1} P), rounded as a
// centred conversion rounds.  l >= 2.
int moddown_rescale_fp(hisa_ctx* ctx, u64* acc, size_t B, int l, const u64* add, u64 add_bs, int add_polys, u64* out);
// Relinearisation of n three-polynomial ciphertexts ([3][l][N], stride words apart) whose division by P is taken
// together with the divScalar by q_{l-1}: out [n][2][l - 1][N] = ((d0, d1) + KS_relin(d2)) / q_{l-1}.
int relinearize_rescale_fp(hisa_ctx* ctx, const u64* cts3, u64 stride, size_t n, int l, u64* out);
int moddown_add_fp(hisa_ctx* ctx, const u64* acc, size_t B, int l, const u64* add, u64 add_bs, int add_polys, u64 add_galois,
                   u64* out, double* y2_ws = nullptr);
// exact integer nearest to the double v (ties away from zero), reduced modulo q
u64 double_to_residue(double v, u64 q);

// Optional per-kernel timing with HIP events on the launch stream (off by default; the benchmark
// turns it on for a separate pass).  One scope brackets one kernel launch.
void prof_begin(const char* kernel, hipStream_t st);
void prof_end(hipStream_t st);
extern bool g_prof_on;

// Analysis backend (Sec. "Compiler": the analyser runs the circuit on a HISA backend that records instead of
// computing).  While a context is in analysis mode every launch wrapper returns at once (no kernel runs; memory is
// still allocated, so handles, levels and scales evolve as in a real run) and the primitives count themselves here.
struct Analysis {
    hisa_op_counts c = {};
    std::set<int32_t> steps;    // left-rotation amounts that needed a key
};
extern thread_local Analysis* t_analysis;   // non-null while the calling thread's context is in analysis mode
// n occurrences of an operation on ciphertexts of `limbs` limbs (call only where t_analysis is set)
#define TALLY(field, OP, n, limbs)                                                   \
    do {                                                                             \
        t_analysis->c.field += (uint64_t)(n);                                        \
        t_analysis->c.limb_sum[OP] += (uint64_t)(n) * (uint64_t)(limbs);             \
        t_analysis->c.limb_sq_sum[OP] += (uint64_t)(n) * (uint64_t)(limbs) * (uint64_t)(limbs); \
    } while (0)
#define DRY_RUN_RETURN() do { if (t_analysis) return hipSuccess; } while (0)
struct ProfScope {
    hipStream_t st;
    bool on;
    ProfScope(const char* kernel, hipStream_t s) : st(s), on(g_prof_on) { if (on) prof_begin(kernel, s); }
    ~ProfScope() { if (on) prof_end(st); }
};

// ---- launch wrappers (every one enqueues on `st` and returns hipGetLastError) ----
hipError_t launch_ntt(const NttTables& t, int log_n, u64* data, u64 batch_stride, int n_polys, const PolyMap& map,
                      hipStream_t st);
hipError_t launch_intt(const NttTables& t, int log_n, u64* data, u64 batch_stride, int n_polys, const PolyMap& map,
                       const InttExtra* extra, hipStream_t st);

// ---- fp64 single-launch transforms with fused neighbours (ntt_fp.hip) ----
enum FpMode {
    FP_FWD_PLAIN = 0,      // u64 coefficients in, u64 NTT form out
    FP_INV_PLAIN = 1,      // u64 NTT form in (optionally gathered through sigma_g), u64 coefficients out
    FP_INV_TO_Y = 2,       // as INV_PLAIN, times a per-limb constant, output = centred doubles (input of base conversion)
    FP_FWD_CONV = 3,       // input = fast base conversion of `a` source limbs (centred doubles); NTT form out as lazily
                           // reduced doubles (|v| <= p/2): the extended digits, which only the inner products read
    FP_FWD_CONV_FINAL = 4, // as FWD_CONV, then out = (acc - ntt) * P^-1 (+ addend, optionally through sigma_g), u64
    FP_INV_D_TO_Y = 5,     // as INV_TO_Y for input that already is doubles times the per-limb constant (no gather)
    FP_FWD_CONV_SUB = 6,   // as FWD_CONV, then out = acc - ntt, u64: the conversion table and acc carry the P^-1, acc the addend
    FP_N_MODES = 7
};

struct FpTask {
    int32_t period;                      // tasks per batch entry
    int16_t pos[HISA_MAX_PRIMES];        // limb position of the task's polynomial inside a batch entry (output side)
    int16_t prime[HISA_MAX_PRIMES];      // its prime
    int8_t digit[HISA_MAX_PRIMES];       // base-conversion modes: which FpArgs::dg entry describes its source limbs
};

#define FP_MAX_DIGITS 8  // digits whose conversions one launch can hold
#define FP_MAX_STEPS 32   // rotations per launch of the shared-decomposition path
struct FpArgs {
    const FpPrime* fprimes;
    const double* ftw;
    const double* utw;
    const double* vtw;
    int n_tasks;                       // filled in by the launcher
    const u64* in; u64 in_bs;          // u64 input [batch][..][N]
    u64* out; u64 out_bs;              // u64 output
    double* yout; u64 yout_bs;         // double output (FP_INV_TO_Y)
    int in_pos_shift;                  // input limb position = pos + in_pos_shift
    u64 galois;                        // inverse modes: gather through sigma_g (0 = none)
    const double* post;                // FP_INV_TO_Y: per task entry constant (centred)
    // base conversion (FP_FWD_CONV*)
    const double* y; u64 y_bs;         // [batch][..][N] centred doubles, source limbs at y_pos0 ..
    int y_pos0, conv_a, total;
    const double* hat;                 // [a][total] (D/c_i) mod t, centred
    // Several digits in one launch (each task entry names its digit in FpTask::digit): n_digits > 1 and dg[] filled
    // in by the caller.  n_digits = 0: one digit, the launcher copies y_pos0, conv_a, hat into dg[0].
    int n_digits;
    struct Digit { const double* hat; int y_pos0, conv_a; } dg[FP_MAX_DIGITS];
    double* scratch; int scratch_polys; // one polynomial of doubles per workgroup (at most scratch_polys workgroups)
    int no_pair;                        // one target limb per task whatever the sizes: `scratch` is then never touched
    // final combine (FP_FWD_CONV_FINAL): batch entries are (ciphertext, polynomial) pairs
    const u64* acc; u64 acc_bs; int acc_pos_shift;
    const double* pinv_tab;            // [prime] P^-1 mod q, centred
    const u64* add; u64 add_bs, add_ps; int add_div, add_polys;  // addend of entry b: add + (b / add_div) * add_bs +
    u64 add_galois;                                              // (b % add_div) * add_ps, if b % add_div < add_polys
    // several rotations of the same step_B ciphertexts in one launch (entries ordered rotation-major): entry b's
    // addend is that of ciphertext (b / add_div) % step_B, gathered through galois_tab[(b / add_div) / step_B];
    // step_B = 0: one rotation, add_galois applies
    int step_B;
    uint32_t galois_tab[FP_MAX_STEPS];
};
hipError_t launch_ntt_fp(int mode, int log_n, const FpArgs& a, const FpTask& tk, u64 n_batch, hipStream_t st);
// workgroups of the transform kernel that the chip holds at once (about: 16 waves per compute unit)
u64 fp_resident_workgroups(int log_n);
// estimated time of one base-conversion launch (conv_a source limbs, `period` target limbs per batch entry), in units
// of one single-target task: rounds of workgroups times the task's relative cost, for the cheaper of the two forms
double fp_conversion_cost(int log_n, int conv_a, int period, u64 n_batch, bool* paired);

// acc[b][p][x] = sum_j e_j[x] * key[j][p][prime(x)] in fp64; e_j[x] comes from ext unless x lies in digit j, then
// from own_src (the NTT-form input itself, read through sigma_g when galois != 0)
hipError_t launch_inner_product_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                   int alpha, const u64* key, int total, const u64* own_src, u64 own_bs, u64 galois,
                                   int gather_ext, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st);
// The same with the elementwise ends of the ModDown folded in (this kernel waits for memory, the transforms for the
// vector ALU).  On the limbs of q:   acc = sum * P^-1 + addend  (canonical residues; addend [batch][add_polys][l][N],
// read through sigma_g like the own-digit limbs, null for none), so that the last kernel only subtracts its transform;
// on the special limbs:  acc = sum * (P/p_m)^-1  as lazily reduced doubles, the input of FP_INV_D_TO_Y.
// pin_tab: [prime] P^-1 mod q_i; post_p: [K] (P/p_m)^-1 mod p_m; both centred doubles.
struct IpFold {
    const double* pin_tab;
    const double* post_p;
    const u64* add; u64 add_bs, add_ps; int add_polys;
};
hipError_t launch_inner_product_fold_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                        int alpha, const u64* key, int total, const u64* own_src, u64 own_bs, u64 galois,
                                        int gather_ext, u64* acc, u64 acc_bs, u64 n_batch, int log_n, const IpFold& fold,
                                        hipStream_t st);
// The same for n_steps rotations of the same n_batch ciphertexts (extended digits computed once from the unrotated
// polynomial): rotation s uses keys[s] and gathers through galois[s]; acc entries are ordered rotation-major.
// c0_src (with pmod[i] = P mod q_i): the b accumulator also takes P * sigma_s(c0) on the limbs of q, c0 read at
// c0_src + b * own_bs like the own-digit limbs.
struct IpSteps {
    const u64* key[FP_MAX_STEPS];
    uint32_t galois[FP_MAX_STEPS];
};
hipError_t launch_inner_product_steps_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                         int alpha, const IpSteps& steps, int n_steps, int total, const u64* own_src,
                                         u64 own_bs, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st,
                                         const u64* c0_src = nullptr, const u64* pmod = nullptr);

// The sum over n_steps rotations of different ciphertexts: ext / own_src entry s * n_batch + b is term s of output b
// (digits from the unrotated polynomial); acc[b] = sum_s sum_j sigma_s(e_j) * key_s[j] on the l + K limbs.
hipError_t launch_inner_product_sum_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                       int alpha, const IpSteps& steps, int n_steps, int total, const u64* own_src, u64 own_bs,
                                       u64* acc, u64 acc_bs, u64 n_batch, int shared_input, int log_n, hipStream_t st);

// sampling (counter-based generator, both sides of the parity tests implement it)
hipError_t launch_sample_uniform(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr, const PolyMap& map, int n_polys,
                                 u64 batch_stride, u64 ctr_step, u64* out, int log_n, hipStream_t st);
hipError_t launch_sample_small(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr, int noise_on, int ternary,
                               const u64* cdt, int cdt_n, const PolyMap& map, int n_polys, u64 batch_stride, u64 ctr_step,
                               u64* out, i64* raw, int log_n, hipStream_t st);

// element-wise kernels over [batch][polys][limbs][N]
enum ElemOp { OP_ADD = 0, OP_SUB = 1 };
hipError_t launch_addsub(const PrimeConst* primes, const u64* a, const u64* b, u64* out, int op, int limbs, int polys_a,
                         int polys_b, u64 n_batch, u64 a_bs, u64 b_bs, u64 o_bs, int log_n, hipStream_t st);
hipError_t launch_add_const(const PrimeConst* primes, const u64* a, u64* out, const u64* consts, int op, int limbs,
                            int polys, int log_n, hipStream_t st);
// entry b is multiplied by plaintext b % pt_period of the pt_period plaintexts at pt
hipError_t launch_mul_plain(const PrimeConst* primes, const u64* a, const u64* pt, u64* out, int limbs, int polys,
                            u64 n_batch, u64 a_bs, u64 o_bs, int log_n, hipStream_t st, unsigned pt_period = 1);
hipError_t launch_mul_const(const PrimeConst* primes, const u64* a, u64* out, const u64* consts, int limbs, int polys,
                            int log_n, hipStream_t st);
hipError_t launch_mul_no_relin(const PrimeConst* primes, const u64* a, const u64* b, u64* out, int limbs, u64 n_batch,
                               u64 a_bs, u64 b_bs, u64 o_bs, int log_n, hipStream_t st);
hipError_t launch_encrypt_combine(const PrimeConst* primes, const u64* secret, const u64* pt, const u64* e, u64* ct,
                                  int limbs, u64 n_batch, u64 pt_bs, int log_n, hipStream_t st);
hipError_t launch_decrypt(const PrimeConst* primes, const u64* secret, const u64* ct, u64* pt, int limbs, int polys,
                          int log_n, hipStream_t st);
hipError_t launch_key_combine(const PrimeConst* primes, const u64* secret, const u64* target, const u64* e,
                              const u64* pmod_all, u64* key_digit, int total, int L, int alpha, int digit, int log_n,
                              hipStream_t st);
hipError_t launch_pointwise_square(const PrimeConst* primes, const u64* s, u64* out, int total, int log_n, hipStream_t st);
hipError_t launch_automorph_ntt(const u64* in, u64 in_bs, u64* out, u64 out_bs, u64 galois, int n_polys, u64 n_batch,
                                int log_n, hipStream_t st);
#define GALOIS_TAB_MAX 256
struct GaloisTab { uint32_t g[GALOIS_TAB_MAX]; };
// several automorphisms of the same inputs: out entry (s, b) = sigma_{tab.g[s]}(in entry b), entries out_bs words apart
hipError_t launch_automorph_steps(const u64* in, u64 in_bs, u64* out, u64 out_bs, const GaloisTab& tab, int n_steps,
                                  int n_polys, u64 n_batch, int log_n, hipStream_t st);
// out[b] = (plain[b].c0 + sum_s sigma_{tab.g[s]}(rot[s * n_batch + b].c0), plain[b].c1) on l limbs; plain may be null;
// shared_input: every term of output b is rot[b]
hipError_t launch_automorph_sum(const PrimeConst* primes, const u64* rot, u64 rot_bs, int n_rot, const GaloisTab& tab,
                                const u64* plain, u64 plain_bs, u64* out, u64 out_bs, u64 n_batch, int shared_input, int l,
                                int log_n, hipStream_t st);
// acc entries (ciphertext, polynomial), acc_bs apart: acc += P * add on the first l limbs, for polynomials < add_polys
hipError_t launch_fold_addend(const PrimeConst* primes, u64* acc, u64 acc_bs, const u64* add, u64 add_bs, u64 add_ps,
                              int add_polys, const u64* pmod, u64 n_cts, int l, int log_n, hipStream_t st);
hipError_t launch_reduce_i64(const PrimeConst* primes, const i64* coeffs, u64* out, int limbs, int n_pts, int log_n,
                             hipStream_t st);
// the same with the output entries out_limbs limbs apart (residues on a second list of primes go behind the first)
hipError_t launch_reduce_i64(const PrimeConst* primes, const i64* coeffs, u64* out, int limbs, int out_limbs, int n_pts,
                             int log_n, hipStream_t st);

// Fast base conversion (centred): for every batch entry and target,
//   out[target] = ( sum_i y[src_pos0+i] * hat[i][prime(target)]  -  #{i : y_i > c_i/2} * D ) mod t
// with y_i the source residues already multiplied by (D/c_i)^-1 mod c_i.
struct ConvArgs {
    const u64* y;      // [batch][..][N], coefficient form
    u64 y_bs;
    int src_pos0;      // first source limb position inside a batch entry of y
    int src_prime0;    // its prime index
    int a;             // number of source limbs
    const u64* hat;    // [a][total]
    const u64* dmod;   // [total]
    int total;
    u64* out;          // [batch][..][N]
    u64 out_bs;
    int n_targets;
    int16_t tgt_pos[HISA_MAX_PRIMES];   // limb position inside a batch entry of out
    int16_t tgt_prime[HISA_MAX_PRIMES];
};
hipError_t launch_base_conv(const PrimeConst* primes, const ConvArgs& args, u64 n_batch, int log_n, hipStream_t st);

// acc[b][p][x] = sum_j ext[b][j][x] * key[j][p][prime(x)], x over l + K limbs (prime(x) = x for x < l, L + x - l above)
hipError_t launch_inner_product(const PrimeConst* primes, const u64* ext, u64 ext_bs, int digits, int l, int K, int L,
                                const u64* key, int total, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st);
// out[b][p][i] = (acc[b][p][i] - conv[b][p][i]) * P^-1 + add[b][p][i]   (p < add_polys; through sigma_g if galois != 0)
hipError_t launch_moddown_final(const PrimeConst* primes, const u64* acc, u64 acc_bs, const u64* conv, u64 conv_bs,
                                const u64* pinv, const u64* pinv_sh, const u64* add, u64 add_bs, int add_polys, u64 galois,
                                u64* out, u64 out_bs, int l, int K, u64 n_batch, int log_n, hipStream_t st);
hipError_t launch_copy_limbs(const u64* src, u64 src_bs, u64* dst, u64 dst_bs, int limbs, u64 n_batch, int log_n,
                             hipStream_t st);

// rescale pieces: r[bp][i] = centred remainder of the last limb modulo q_i; out = (ct - NTT(r)) * q_last^-1
hipError_t launch_rescale_spread(const PrimeConst* primes, const u64* last, u64* r, int l, u64 n_bp, int log_n,
                                 hipStream_t st);
hipError_t launch_rescale_final(const PrimeConst* primes, const u64* ct, const u64* r, const u64* qlinv, const u64* qlinv_sh,
                                u64* out, int l, u64 n_bp, int log_n, hipStream_t st);

// encode / decode
hipError_t launch_encode(const double* cs, const double* sn, const uint32_t* g, const double* re, const double* im,
                         int count, int n_pts, double factor, i64* coeffs, int log_n, hipStream_t st);
// piecewise-constant plaintexts: indicator encodings of nb slot sets (g[set_begin[b] .. set_begin[b+1]) lists 5^slot
// mod 2N of set b), then coeffs[p] = round(factor * sum_b v[p][b] * basis[b])
hipError_t launch_encode_basis(const double* cs, const uint32_t* g, const int* set_begin, int nb, double* basis, int log_n,
                               hipStream_t st);
hipError_t launch_encode_combine(const double* basis, int nb, const double* v, int n_pts, double factor, i64* coeffs,
                                 int log_n, hipStream_t st);
// the same maps through the O(N log N) transform over the slot order (encode.hip); pow5: [N/2] 5^j mod 2N
hipError_t launch_decode_fft(const double* cs, const double* sn, const uint32_t* pow5, const double* m, int count, void* work,
                             double* re, double* im, int log_n, hipStream_t st);
hipError_t launch_encode_fft(const double* cs, const double* sn, const uint32_t* pow5, const double* re, const double* im,
                             const uint32_t* slots, int count, int n_pts, double factor, void* work, i64* coeffs, int log_n,
                             hipStream_t st);
hipError_t launch_crt_to_double(const PrimeConst* primes, const u64* coeff_form, int limbs, const u64* garner_inv,
                                const u64* garner_inv_sh, int L, double inv_scale, double* out, int log_n, hipStream_t st);
hipError_t launch_decode(const double* cs, const double* sn, const double* m, int count, double* re, double* im, int log_n,
                         hipStream_t st);
