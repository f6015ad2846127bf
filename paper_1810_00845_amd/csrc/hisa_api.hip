// Host side of libhisa: context set-up (primes, roots, tables, keys), handle
// and device-memory management, argument checks, and the launch sequences
// behind every C-ABI entry point.  No arithmetic on polynomial data happens
// here; the kernels are in ntt.hip, elementwise.hip, keyswitch.hip, encode.hip.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>

#include "hisa_internal.hpp"

// ---------------------------------------------------------------------------
// host-side number theory (set-up only)
// ---------------------------------------------------------------------------
namespace hm {
static inline u64 mul(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
static u64 pw(u64 b, u64 e, u64 m) {
    u64 r = 1 % m;
    b %= m;
    for (; e; e >>= 1, b = mul(b, b, m))
        if (e & 1) r = mul(r, b, m);
    return r;
}
static inline u64 inv(u64 a, u64 p) { return pw(a % p, p - 2, p); }
static inline u64 shoup(u64 w, u64 q) { return (u64)(((u128)w << 64) / q); }

// deterministic Miller-Rabin for 64-bit inputs (witnesses: the primes up to 37)
static bool is_prime(u64 n) {
    const u64 wit[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return false;
    for (u64 w : wit) {
        if (n == w) return true;
        if (n % w == 0) return false;
    }
    u64 odd = n - 1;
    int twos = 0;
    while (!(odd & 1)) { odd >>= 1; ++twos; }
    for (u64 w : wit) {
        u64 x = pw(w, odd, n);
        if (x == 1 || x == n - 1) continue;
        bool witness = true;
        for (int k = 1; k < twos && witness; ++k) {
            x = mul(x, x, n);
            if (x == n - 1) witness = false;
        }
        if (witness) return false;
    }
    return true;
}

// largest unused prime = 1 (mod 2N) below 2^bits
static u64 pick_prime(unsigned bits, unsigned log_n, const std::vector<u64>& taken) {
    const u64 step = (u64)2 << log_n;
    for (u64 c = ((u64)1 << bits) + 1 - step; c > step; c -= step) {
        if (!is_prime(c)) continue;
        if (std::find(taken.begin(), taken.end(), c) == taken.end()) return c;
    }
    return 0;
}

// primitive 2N-th root of unity from the smallest base that works
static u64 find_psi(u64 q, unsigned log_n) {
    const u64 n = (u64)1 << log_n;
    for (u64 base = 2; base < q; ++base) {
        u64 cand = pw(base, (q - 1) / (2 * n), q);
        if (pw(cand, n, q) == q - 1) return cand;
    }
    return 0;
}

static inline uint32_t brev(uint32_t x, unsigned bits) {
    uint32_t r = 0;
    for (unsigned i = 0; i < bits; ++i) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

// exact integer nearest to the double v (ties away from zero), reduced modulo q
static u64 double_to_residue(double v, u64 q) {
    bool neg = v < 0;
    double a = fabs(v);
    u64 r;
    if (a < 9007199254740992.0) {  // below 2^53: round() is exact
        r = (u64)round(a) % q;
    } else {                        // an integer already: mantissa * 2^e
        int e;
        double m = frexp(a, &e);    // a = m * 2^e, m in [0.5, 1)
        u64 mant = (u64)ldexp(m, 53);
        r = mul(mant % q, pw(2, (u64)(e - 53), q), q);
    }
    return (neg && r) ? q - r : r;
}
}  // namespace hm

u64 double_to_residue(double v, u64 q) { return hm::double_to_residue(v, q); }

// ---------------------------------------------------------------------------
// per-kernel timing (HIP events on the launch stream)
// ---------------------------------------------------------------------------
bool g_prof_on = false;
thread_local Analysis* t_analysis = nullptr;
namespace {
struct ProfRec { std::string kernel; hipEvent_t t0, t1; };
std::vector<ProfRec> g_prof_recs;
}
void prof_begin(const char* kernel, hipStream_t st) {
    ProfRec r{kernel, nullptr, nullptr};
    if (hipEventCreate(&r.t0) != hipSuccess || hipEventCreate(&r.t1) != hipSuccess) return;
    (void)hipEventRecord(r.t0, st);
    g_prof_recs.push_back(r);
}
void prof_end(hipStream_t st) {
    if (!g_prof_recs.empty()) (void)hipEventRecord(g_prof_recs.back().t1, st);
}

extern "C" int hisa_profile_enable(hisa_ctx* ctx, int on) {
    if (!ctx) return HISA_ERR_ARG;
    g_prof_on = on != 0;
    return HISA_OK;
}

// Writes one line per kernel: "<name>\t<launches>\t<total ms>\n" into host_buf and clears the records.
extern "C" int hisa_profile_read(hisa_ctx* ctx, char* host_buf, size_t cap) {
    if (!ctx || !host_buf || cap == 0) return HISA_ERR_ARG;
    (void)hipStreamSynchronize(ctx->stream);
    std::map<std::string, std::pair<long, double>> agg;
    for (auto& r : g_prof_recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.t0, r.t1) == hipSuccess) {
            agg[r.kernel].first += 1;
            agg[r.kernel].second += ms;
        }
        (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
    }
    g_prof_recs.clear();
    std::string out;
    char line[256];
    for (auto& kv : agg) {
        snprintf(line, sizeof line, "%s\t%ld\t%.6f\n", kv.first.c_str(), kv.second.first, kv.second.second);
        out += line;
    }
    if (out.size() + 1 > cap) return HISA_ERR_ARG;
    memcpy(host_buf, out.c_str(), out.size() + 1);
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// errors, memory
// ---------------------------------------------------------------------------
// Intermediates of hisa_rot_left_noalloc (conversion input, extended digits, accumulators, ModDown input of ONE
// ciphertext).  Every GPU holds its own copy of this array for the life of the process.  `scratch` is only a
// host-side stand-in for it: its device address on a given GPU is asked for once per device (scratch_address, at
// hisa_create, with that device current) and that pointer is what host code hands to kernels.
static __device__ __align__(256) unsigned char scratch[HISA_NOALLOC_SCRATCH_BYTES];
#define HISA_MAX_DEVICES 64
static void* g_scratch_ptr[HISA_MAX_DEVICES];

// device address of `scratch` on the current device
static int scratch_address(hisa_ctx* ctx, int* device, void** ptr) {
    int dev = -1;
    HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev < 0 || dev >= HISA_MAX_DEVICES) return fail(ctx, HISA_ERR_HIP, "device ordinal %d out of range", dev);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(ctx, hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ctx, HISA_ERR_HIP, "no device address for the static scratch array");
        g_scratch_ptr[dev] = p;
    }
    *device = dev;
    *ptr = g_scratch_ptr[dev];
    return HISA_OK;
}
int fail(hisa_ctx* ctx, int code, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return code;
}

DevBlock* dev_alloc(hisa_ctx* ctx, size_t bytes) {
    bytes = (bytes + 255) & ~(size_t)255;
    if (bytes == 0) bytes = 256;
    void* p = nullptr;
    auto it = ctx->pool.find(bytes);
    if (it != ctx->pool.end() && !it->second.empty()) {
        p = it->second.back();
        it->second.pop_back();
    } else {
        if (hipMalloc(&p, bytes) != hipSuccess) {
            (void)hipGetLastError();
            // give cached blocks back and retry once
            for (auto& kv : ctx->pool) {
                for (void* q : kv.second) (void)hipFree(q);
                kv.second.clear();
            }
            if (hipMalloc(&p, bytes) != hipSuccess) {
                (void)hipGetLastError();
                fail(ctx, HISA_ERR_OOM, "device allocation of %zu bytes failed", bytes);
                return nullptr;
            }
        }
        ctx->pool_bytes += bytes;
    }
    DevBlock* b = new DevBlock{p, bytes, 1};
    ctx->live[(uintptr_t)p] = bytes;
    return b;
}

u64 dev_words_behind(const hisa_ctx* ctx, const void* p) {
    const uintptr_t a = (uintptr_t)p;
    auto it = ctx->live.upper_bound(a);
    if (it == ctx->live.begin()) return 0;
    --it;
    if (a >= it->first + it->second) return 0;
    return (u64)(it->first + it->second - a) / sizeof(u64);
}

// Work on one stream: a block returned to the pool may be handed out again at
// once, later kernels are ordered behind the earlier ones that used it.
void dev_release(hisa_ctx* ctx, DevBlock* b) {
    if (!b) return;
    if (--b->refs > 0) return;
    ctx->live.erase((uintptr_t)b->ptr);
    ctx->pool[b->bytes].push_back(b->ptr);
    delete b;
}



// n ciphertext handles that are views of one allocation, [n][polys][limbs][N]
int alloc_ct_batch(hisa_ctx* ctx, size_t n, uint32_t polys, uint32_t limbs, double scale, hisa_ct** out) {
    size_t words = ct_words(ctx, polys, limbs);
    DevBlock* blk = dev_alloc(ctx, n * words * sizeof(u64));
    if (!blk) return HISA_ERR_OOM;
    blk->refs = (int)n;
    for (size_t i = 0; i < n; i++)
        out[i] = new hisa_ct{HISA_MAGIC_CT, blk, (u64*)blk->ptr + i * words, polys, limbs, scale};
    if (t_analysis && n && (t_analysis->c.min_limbs == 0 || limbs < t_analysis->c.min_limbs)) t_analysis->c.min_limbs = limbs;
    return HISA_OK;
}

int alloc_pt(hisa_ctx* ctx, uint32_t limbs, double scale, hisa_pt** out) {
    DevBlock* blk = dev_alloc(ctx, (size_t)limbs * ctx->N * sizeof(u64));
    if (!blk) return HISA_ERR_OOM;
    *out = new hisa_pt{HISA_MAGIC_PT, blk, (u64*)blk->ptr, limbs, scale};
    return HISA_OK;
}

int gather_batch(hisa_ctx* ctx, const hisa_ct* const* cts, size_t n, BatchIn* bi) {
    const size_t words = ct_words(ctx, cts[0]->polys, cts[0]->limbs);
    bool even = true;
    // views of ONE allocation only: separately allocated ciphertexts can be neighbours in the address space, and a
    // device-to-device copy over the whole batch must not cross an allocation boundary
    for (size_t i = 1; i < n && even; i++) even = cts[i]->blk == cts[0]->blk && cts[i]->data == cts[0]->data + i * words;
    if (even) {
        bi->base = cts[0]->data;
        bi->stride = words;
        return HISA_OK;
    }
    bi->tmp = dev_alloc(ctx, n * words * sizeof(u64));
    if (!bi->tmp) return HISA_ERR_OOM;
    // one copy per run of neighbouring views of one allocation (a concatenation of two batches is two runs)
    for (size_t i = 0; i < n;) {
        size_t j = i + 1;
        while (j < n && cts[j]->blk == cts[i]->blk && cts[j]->data == cts[i]->data + (j - i) * words) j++;
        HIP_TRY(ctx, hipMemcpyAsync((u64*)bi->tmp->ptr + i * words, cts[i]->data, (j - i) * words * sizeof(u64),
                                    hipMemcpyDeviceToDevice, ctx->stream));
        i = j;
    }
    bi->base = (u64*)bi->tmp->ptr;
    bi->stride = words;
    return HISA_OK;
}

int check_batch_shape(hisa_ctx* ctx, const hisa_ct* const* cts, size_t n, uint32_t polys) {
    if (!cts || n == 0) return fail(ctx, HISA_ERR_ARG, "empty batch");
    for (size_t i = 0; i < n; i++) {
        if (!valid_ct(cts[i])) return fail(ctx, HISA_ERR_ARG, "batch entry %zu is not a ciphertext", i);
        if (cts[i]->limbs != cts[0]->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "batch entries differ in level");
        if (cts[i]->polys != cts[0]->polys || (polys && cts[i]->polys != polys))
            return fail(ctx, HISA_ERR_SIZE, "batch entry %zu has %u polynomials", i, cts[i]->polys);
    }
    return HISA_OK;
}

PolyMap identity_map(int limbs) {
    PolyMap m = {};
    m.period = limbs;
    for (int i = 0; i < limbs; i++) m.prime_of[i] = (int16_t)i;
    return m;
}

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
template <class T>
static hipError_t upload(T** dst, const std::vector<T>& src) {
    hipError_t e = hipMalloc((void**)dst, src.size() * sizeof(T));
    if (e != hipSuccess) return e;
    return hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
}

static double centred_double(u64 x, u64 q) { return x > q / 2 ? -(double)(q - x) : (double)x; }

static void build_conv_table_host(const hisa_ctx* ctx, const std::vector<int>& src, std::vector<u64>& inv_hat,
                                  std::vector<u64>& inv_hat_sh, std::vector<u64>& hat, std::vector<u64>& dmod) {
    const int a = (int)src.size(), total = (int)ctx->total;
    inv_hat.assign(a, 0); inv_hat_sh.assign(a, 0); hat.assign((size_t)a * total, 0); dmod.assign(total, 0);
    for (int i = 0; i < a; i++) {
        const u64 ci = ctx->mod[src[i]];
        u64 prod = 1 % ci;
        for (int m = 0; m < a; m++)
            if (m != i) prod = hm::mul(prod, ctx->mod[src[m]] % ci, ci);
        inv_hat[i] = hm::inv(prod, ci);
        inv_hat_sh[i] = hm::shoup(inv_hat[i], ci);
        for (int t = 0; t < total; t++) {
            const u64 qt = ctx->mod[t];
            u64 h = 1 % qt;
            for (int m = 0; m < a; m++)
                if (m != i) h = hm::mul(h, ctx->mod[src[m]] % qt, qt);
            hat[(size_t)i * total + t] = h;
        }
    }
    for (int t = 0; t < total; t++) {
        const u64 qt = ctx->mod[t];
        u64 d = 1 % qt;
        for (int m = 0; m < a; m++) d = hm::mul(d, ctx->mod[src[m]] % qt, qt);
        dmod[t] = d;
    }
}

static int make_conv_table(hisa_ctx* ctx, const std::vector<int>& src, ConvTable* tab) {
    std::vector<u64> ih, ihs, hat, dmod;
    build_conv_table_host(ctx, src, ih, ihs, hat, dmod);
    tab->a = (int)src.size();
    for (int i = 0; i < tab->a; i++) tab->src[i] = src[i];
    tab->inv_hat = ih;
    HIP_TRY(ctx, upload(&tab->d_inv_hat, ih));
    HIP_TRY(ctx, upload(&tab->d_inv_hat_sh, ihs));
    HIP_TRY(ctx, upload(&tab->d_hat, hat));
    HIP_TRY(ctx, upload(&tab->d_dmod, dmod));
    tab->d_hat_f = nullptr;
    if (ctx->tabs.fp_ok) {
        std::vector<double> hf(hat.size());
        for (int i = 0; i < tab->a; i++)
            for (uint32_t t = 0; t < ctx->total; t++) hf[(size_t)i * ctx->total + t] = centred_double(hat[(size_t)i * ctx->total + t], ctx->mod[t]);
        HIP_TRY(ctx, upload(&tab->d_hat_f, hf));
    }
    return HISA_OK;
}

static void free_conv_table(ConvTable* t) {
    (void)hipFree(t->d_hat_f);
    (void)hipFree(t->d_inv_hat); (void)hipFree(t->d_inv_hat_sh); (void)hipFree(t->d_hat); (void)hipFree(t->d_dmod);
}

// conversion table of digit j restricted to `a` present primes
static int modup_table(hisa_ctx* ctx, int digit, int a, ConvTable** out) {
    auto key = std::make_pair(digit, a);
    auto it = ctx->modup_tabs.find(key);
    if (it == ctx->modup_tabs.end()) {
        std::vector<int> src;
        for (int i = 0; i < a; i++) src.push_back(digit * (int)ctx->alpha + i);
        ConvTable tab = {};
        TRY(make_conv_table(ctx, src, &tab));
        it = ctx->modup_tabs.emplace(key, tab).first;
    }
    *out = &it->second;
    return HISA_OK;
}

static int sample_secret(hisa_ctx* ctx);
static int fp_post_tables(hisa_ctx* ctx, int l, double** post_q, double** post_p, bool lookup_only);
static std::vector<u64> gauss_table(double sigma);

extern "C" int hisa_create(const hisa_params* prm, void* hip_stream, hisa_ctx** out) {
    if (!prm || !out) return HISA_ERR_ARG;
    *out = nullptr;
    if (prm->log_n < 10 || prm->log_n > 16 || prm->num_q < 1 || prm->num_q > HISA_MAX_Q || prm->dnum < 1 ||
        prm->dnum > prm->num_q || prm->noise > 1)
        return HISA_ERR_ARG;
    if (prm->secret_kind > 1 || (prm->secret_kind == 1 && (prm->hamming_weight < 1 || prm->hamming_weight > (1u << prm->log_n))))
        return HISA_ERR_ARG;
    if (prm->sigma != 0.0 && !(prm->sigma > 0.2 && prm->sigma <= 10.0)) return HISA_ERR_ARG;
    const uint32_t alpha = (prm->num_q + prm->dnum - 1) / prm->dnum;
    if (prm->num_q + alpha > HISA_MAX_PRIMES) return HISA_ERR_ARG;
    for (uint32_t i = 0; i < prm->num_q; i++)
        if (prm->q_bits[i] < prm->log_n + 2 || prm->q_bits[i] > 60) return HISA_ERR_ARG;
    if (prm->special_bits < prm->log_n + 2 || prm->special_bits > 60) return HISA_ERR_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return HISA_ERR_HIP;

    hisa_ctx* ctx = new hisa_ctx();
    ctx->prm = *prm;
    ctx->log_n = prm->log_n; ctx->N = 1u << prm->log_n;
    ctx->L = prm->num_q; ctx->dnum = prm->dnum; ctx->alpha = alpha; ctx->K = alpha; ctx->total = ctx->L + ctx->K;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->enc_counter = 0; ctx->pool_bytes = 0; ctx->moddown_tab = nullptr;
    *out = ctx;  // from here on the caller can read last_error and must destroy

    const u64 n = ctx->N;
    for (uint32_t i = 0; i < ctx->total; i++) {
        unsigned bits = i < ctx->L ? prm->q_bits[i] : prm->special_bits;
        u64 p = hm::pick_prime(bits, ctx->log_n, ctx->mod);
        if (!p) return fail(ctx, HISA_ERR_ARG, "no %u-bit prime = 1 mod 2N left", bits);
        ctx->mod.push_back(p);
        ctx->psi.push_back(hm::find_psi(p, ctx->log_n));
    }
    // per-prime constants and twiddle tables
    std::vector<u64> tw((size_t)ctx->total * n), tw_sh(tw.size()), itw(tw.size()), itw_sh(tw.size());
    std::vector<u64> fwd(n), bwd(n);
    for (uint32_t i = 0; i < ctx->total; i++) {
        const u64 q = ctx->mod[i];
        PrimeConst pc;
        pc.q = q;
        u128 ratio = (~(u128)0) / q;  // floor((2^128 - 1)/q) = floor(2^128/q) since q is odd and > 1
        pc.r1 = (u64)(ratio >> 64); pc.r0 = (u64)ratio;
        pc.n_inv = hm::inv(n % q, q); pc.n_inv_sh = hm::shoup(pc.n_inv, q);
        pc.half = q / 2;
        ctx->pc.push_back(pc);
        const u64 psi = ctx->psi[i], psi_inv = hm::inv(psi, q);
        fwd[0] = bwd[0] = 1;
        for (u64 e = 1; e < n; e++) { fwd[e] = hm::mul(fwd[e - 1], psi, q); bwd[e] = hm::mul(bwd[e - 1], psi_inv, q); }
        for (u64 x = 0; x < n; x++) {
            const u64 e = hm::brev((uint32_t)x, ctx->log_n);
            const size_t o = (size_t)i * n + x;
            tw[o] = fwd[e]; tw_sh[o] = hm::shoup(fwd[e], q);
            itw[o] = bwd[e]; itw_sh[o] = hm::shoup(bwd[e], q);
        }
    }
    HIP_TRY(ctx, upload(&ctx->d_primes, ctx->pc));
    HIP_TRY(ctx, upload(&ctx->d_tw, tw));
    HIP_TRY(ctx, upload(&ctx->d_tw_sh, tw_sh));
    HIP_TRY(ctx, upload(&ctx->d_itw, itw));
    HIP_TRY(ctx, upload(&ctx->d_itw_sh, itw_sh));
    ctx->tabs = NttTables{ctx->d_primes, ctx->d_tw, ctx->d_tw_sh, ctx->d_itw, ctx->d_itw_sh, 0, nullptr, nullptr, nullptr, nullptr};
    // fp64 path: every prime below 2^50 and a ring degree the single-launch transform covers
    {
        bool fp_ok = ctx->log_n >= 12 && ctx->log_n <= 15;
        for (u64 q : ctx->mod) fp_ok = fp_ok && q < ((u64)1 << 50);
        if (fp_ok) {
            std::vector<FpPrime> fpr(ctx->total);
            std::vector<double> ftw(tw.size()), utw(tw.size()), vtw(tw.size()), pinv_f(ctx->total, 0.0);
            for (uint32_t i = 0; i < ctx->total; i++) {
                const u64 q = ctx->mod[i];
                fpr[i].p = (double)q; fpr[i].pinv = 1.0 / (double)q; fpr[i].half = (double)(q / 2);
                const u64 psi_inv = hm::inv(ctx->psi[i], q);
                bwd[0] = 1;
                for (u64 e = 1; e < n; e++) bwd[e] = hm::mul(bwd[e - 1], psi_inv, q);   // psi^-e
                const size_t o = (size_t)i * n;
                for (u64 x = 0; x < n; x++) vtw[o + x] = centred_double(hm::mul(bwd[x], ctx->pc[i].n_inv, q), q);
                // forward twiddles psi^bitrev(x), permuted inside each level so that the per-thread part of the index
                // is the fastest one: levels 1..5 (x < 32) as they are; levels 6..10: x = ((32 + a) << j) + g stored at
                // (32 << j) + g * 32 + a; levels 11..: x = ((1024 + T) << j) + g stored at (1024 << j) + g * 1024 + T
                for (u64 x = 0; x < n && x < 32; x++) ftw[o + x] = centred_double(tw[o + x], q);
                for (u64 first : {(u64)32, (u64)1024})
                    for (u64 j = 0; (first << j) < n && (first == 1024 || j < 5); j++)
                        for (u64 g = 0; g < ((u64)1 << j); g++)
                            for (u64 tp = 0; tp < first; tp++)
                                ftw[o + (first << j) + g * first + tp] = centred_double(tw[o + ((first + tp) << j) + g], q);
                utw[o] = 0.0;
                for (u64 m = 1; m < n; m <<= 1)   // psi^(-k N/m), k < m: exponents stay below N
                    for (u64 k = 0; k < m; k++) utw[o + m + k] = centred_double(bwd[k * (n / m)], q);
            }
            HIP_TRY(ctx, upload(&ctx->d_fprimes, fpr));
            HIP_TRY(ctx, upload(&ctx->d_ftw, ftw));
            HIP_TRY(ctx, upload(&ctx->d_utw, utw));
            HIP_TRY(ctx, upload(&ctx->d_vtw, vtw));
            ctx->tabs.fp_ok = 1; ctx->tabs.fprimes = ctx->d_fprimes;
            ctx->tabs.ftw = ctx->d_ftw; ctx->tabs.utw = ctx->d_utw; ctx->tabs.vtw = ctx->d_vtw;
        }
    }

    // mod-down: source = the special primes; P^-1 and P modulo every q_i
    {
        std::vector<int> src;
        for (uint32_t m = 0; m < ctx->K; m++) src.push_back((int)(ctx->L + m));
        ctx->moddown_tab = new ConvTable();
        TRY(make_conv_table(ctx, src, ctx->moddown_tab));
        std::vector<u64> pinv(ctx->L), pinv_sh(ctx->L), pmod(ctx->total, 0);
        for (uint32_t i = 0; i < ctx->total; i++) {
            const u64 q = ctx->mod[i];
            u64 pm = 1 % q;
            for (uint32_t m = 0; m < ctx->K; m++) pm = hm::mul(pm, ctx->mod[ctx->L + m] % q, q);
            pmod[i] = pm;
            if (i < ctx->L) { pinv[i] = hm::inv(pm, q); pinv_sh[i] = hm::shoup(pinv[i], q); }
        }
        HIP_TRY(ctx, upload(&ctx->d_pinv, pinv));
        HIP_TRY(ctx, upload(&ctx->d_pinv_sh, pinv_sh));
        HIP_TRY(ctx, upload(&ctx->d_pmod, pmod));
        if (ctx->tabs.fp_ok) {
            std::vector<double> pf(ctx->total, 0.0);
            for (uint32_t i = 0; i < ctx->L; i++) pf[i] = centred_double(pinv[i], ctx->mod[i]);
            HIP_TRY(ctx, upload(&ctx->d_pinv_f, pf));
            {   // (P/p_m) P^-1 mod q_i: the conversion of FP_FWD_CONV_SUB
                std::vector<u64> ih, ihs, hat, dmod;
                build_conv_table_host(ctx, src, ih, ihs, hat, dmod);
                std::vector<double> hp((size_t)ctx->K * ctx->total, 0.0);
                for (uint32_t m = 0; m < ctx->K; m++)
                    for (uint32_t i = 0; i < ctx->L; i++)
                        hp[(size_t)m * ctx->total + i] = centred_double(hm::mul(hat[(size_t)m * ctx->total + i], pinv[i], ctx->mod[i]), ctx->mod[i]);
                HIP_TRY(ctx, upload(&ctx->d_moddown_hat_pin, hp));
            }
            ctx->fp_scratch_polys = ctx->log_n <= 13 ? 1024 : 512;
            HIP_TRY(ctx, hipMalloc(&ctx->d_fp_scratch, (size_t)ctx->fp_scratch_polys * ctx->N * sizeof(double)));
        }
    }
    // 2N-th roots of unity for encode / decode
    {
        std::vector<double> cs(2 * n), sn(2 * n);
        const long double pi = 3.14159265358979323846264338327950288L;
        for (u64 t = 0; t < 2 * n; t++) {
            cs[t] = (double)cosl(pi * (long double)t / (long double)n);
            sn[t] = (double)sinl(pi * (long double)t / (long double)n);
        }
        HIP_TRY(ctx, upload(&ctx->d_cos, cs));
        HIP_TRY(ctx, upload(&ctx->d_sin, sn));
        std::vector<uint32_t> pow5(n / 2);
        uint32_t g = 1;
        for (u64 j = 0; j < n / 2; j++) { pow5[j] = g; g = (g * 5u) & (uint32_t)(2 * n - 1); }
        HIP_TRY(ctx, upload(&ctx->d_pow5, pow5));
    }
    {
        const std::vector<u64> cdt = gauss_table(prm->sigma == 0.0 ? 3.2 : prm->sigma);
        ctx->gauss_cdt_n = (int)cdt.size();
        HIP_TRY(ctx, upload(&ctx->d_gauss_cdt, cdt));
    }
    HIP_TRY(ctx, hipMalloc((void**)&ctx->d_secret, (size_t)ctx->total * n * sizeof(u64)));
    TRY(sample_secret(ctx));
    TRY(scratch_address(ctx, &ctx->device, &ctx->noalloc_ws));
    if (ctx->tabs.fp_ok && ctx->dnum <= 8) {
        // the small per-level tables of the fused key switch, so that no later call has to build (and allocate) one
        double *pq, *pp;
        for (uint32_t l = 1; l <= ctx->L; l++) TRY(fp_post_tables(ctx, (int)l, &pq, &pp, false));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_destroy(hisa_ctx* ctx) {
    if (!ctx) return HISA_OK;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->analysis) {
        if (t_analysis == ctx->analysis) t_analysis = nullptr;
        delete ctx->analysis;
    }
    for (auto* m : {&ctx->keys, &ctx->aux})
        for (auto& kv : *m)
            if (kv.second.blk) { (void)hipFree(kv.second.blk->ptr); delete kv.second.blk; }
    for (auto& kv : ctx->pool)
        for (void* p : kv.second) (void)hipFree(p);
    for (auto& kv : ctx->modup_tabs) free_conv_table(&kv.second);
    if (ctx->moddown_tab) { free_conv_table(ctx->moddown_tab); delete ctx->moddown_tab; }
    (void)hipFree(ctx->d_primes); (void)hipFree(ctx->d_tw); (void)hipFree(ctx->d_tw_sh); (void)hipFree(ctx->d_itw);
    (void)hipFree(ctx->d_itw_sh); (void)hipFree(ctx->d_secret); (void)hipFree(ctx->d_pinv); (void)hipFree(ctx->d_pinv_sh);
    (void)hipFree(ctx->d_fprimes); (void)hipFree(ctx->d_ftw); (void)hipFree(ctx->d_utw); (void)hipFree(ctx->d_vtw);
    (void)hipFree(ctx->d_pinv_f); (void)hipFree(ctx->d_moddown_hat_pin);
    (void)hipFree(ctx->d_fp_scratch);
    (void)hipFree(ctx->d_pmod); (void)hipFree(ctx->d_cos); (void)hipFree(ctx->d_sin); (void)hipFree(ctx->d_pow5);
    (void)hipFree(ctx->d_gauss_cdt);
    delete ctx;
    return HISA_OK;
}

extern "C" const char* hisa_last_error(const hisa_ctx* ctx) { return ctx ? ctx->err.c_str() : "no context"; }

extern "C" int hisa_sync(hisa_ctx* ctx) {
    if (!ctx) return HISA_ERR_ARG;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// keys
// ---------------------------------------------------------------------------
// The generator of all randomness on the host (the kernels hold the device form): two rounds of a 64-bit mixer,
// the first over seed and stream (kind, counter), the second over the index.
static u64 host_mix(u64 x) {
    x ^= x >> 32; x *= 0x6a09e667f3bcc909ULL;
    x ^= x >> 29; x *= 0xbb67ae8584caa73bULL;
    return x ^ (x >> 32);
}
static u64 host_rnd(u64 seed, u64 kind, u64 ctr, u64 idx) {
    const u64 step = 0x3c6ef372fe94f82bULL;
    return host_mix(host_mix(seed + step * (((kind << 56) | ctr) + 1)) + step * (idx + 1));
}

// Cumulative table of the error distribution: entry k = floor(2^63 * P(|X| <= k)), k < floor(6 sigma), for the pmf
// proportional to exp(-x^2 / (2 sigma^2)) cut at |x| <= floor(6 sigma).  For sigma = 3.2 the entries are constants
// (computed once with 80 digits); for any other sigma they are computed here in extended precision, by running sums
// from x = 0 upwards, which places them within a few units of 2^-63 of the exact values.
static std::vector<u64> gauss_table(double sigma) {
    static const u64 table_3_2[19] = {
        1149872836518706973ULL, 3340023669317320718ULL, 5231742859181312982ULL, 6713673040852152709ULL,
        7766573333558595572ULL, 8445050410543775182ULL, 8841576294031517592ULL, 9051758687454227207ULL,
        9152802460441190481ULL, 9196859083481262423ULL, 9214281214904026344ULL, 9220529772758650828ULL,
        9222562348483741346ULL, 9223162004373033245ULL, 9223322456656299389ULL, 9223361395058736926ULL,
        9223369965413244325ULL, 9223371676247247624ULL, 9223371985993021523ULL};
    if (sigma == 3.2) return std::vector<u64>(table_3_2, table_3_2 + 19);
    const int cut = (int)floor(6.0 * sigma);
    const long double denom = 2.0L * (long double)sigma * (long double)sigma;
    std::vector<long double> run((size_t)cut + 1);
    for (int x = 0; x <= cut; x++) {
        const long double w = expl(-((long double)x * (long double)x) / denom);
        run[x] = x ? run[x - 1] + 2.0L * w : w;
    }
    std::vector<u64> t((size_t)cut);
    for (int k = 0; k < cut; k++) {
        const long double v = floorl(ldexpl(run[k] / run[cut], 63));
        t[k] = v >= 9223372036854775807.0L ? 9223372036854775807ULL : (u64)v;
    }
    return t;
}

// The secret, NTT form over all primes.  Uniform ternary: one word per coefficient, drawn by the sampling kernel.
// Fixed Hamming weight h: a partial shuffle of the positions 0..N-1 on the host (h dependent steps: step i draws
// word i of the secret's stream, exchanges entry i of the permutation with entry i + (word >> 1) mod (N - i), and
// gives the coefficient now at entry i the sign of the word's low bit), reduced and transformed on the GPU.
static int sample_secret(hisa_ctx* ctx) {
    PolyMap all = identity_map((int)ctx->total);
    if (ctx->prm.secret_kind == 1) {
        const u64 n = ctx->N;
        std::vector<u64> perm(n);
        for (u64 j = 0; j < n; j++) perm[j] = j;
        ctx->sparse_secret.assign(n, 0);
        for (u64 i = 0; i < ctx->prm.hamming_weight; i++) {
            const u64 u = host_rnd(ctx->prm.seed, 1, 0, i);
            std::swap(perm[i], perm[i + (u >> 1) % (n - i)]);
            ctx->sparse_secret[perm[i]] = (u & 1) ? -1 : 1;
        }
        Temp co(ctx, n * sizeof(i64));
        if (!co.ok()) return HISA_ERR_OOM;
        HIP_TRY(ctx, hipMemcpyAsync(co.blk->ptr, ctx->sparse_secret.data(), n * sizeof(i64), hipMemcpyHostToDevice, ctx->stream));
        HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co.as<i64>(), ctx->d_secret, (int)ctx->total, 1, (int)ctx->log_n, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));   // the host vector is pageable memory
    } else {
        HIP_TRY(ctx, launch_sample_small(ctx->d_primes, ctx->prm.seed, 1, 0, 0, 1, nullptr, 0, all, 1, 0, 0, ctx->d_secret, nullptr,
                                         (int)ctx->log_n, ctx->stream));
    }
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, ctx->d_secret, 0, (int)ctx->total, all, ctx->stream));
    return HISA_OK;
}

// key towards `target` (NTT form over all primes): per digit, a uniform (kind 4), e Gaussian (kind 5),
// b = -a*s + e + [prime in digit] (P mod q) target
static int fill_switch_key(hisa_ctx* ctx, u64 key_id, const u64* target, const SwitchKey& key) {
    const size_t n = ctx->N, total = ctx->total;
    Temp e(ctx, total * n * sizeof(u64));
    if (!e.ok()) return HISA_ERR_OOM;
    PolyMap all = identity_map((int)total);
    for (uint32_t j = 0; j < ctx->dnum; j++) {
        const u64 ctr = (key_id << 8) | j;
        u64* digit = key.data + (size_t)j * 2 * total * n;
        HIP_TRY(ctx, launch_sample_uniform(ctx->d_primes, ctx->prm.seed, 4, ctr, all, (int)total, 0, 0, digit + total * n,
                                           (int)ctx->log_n, ctx->stream));
        HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, digit + total * n, 0, (int)total, all, ctx->stream));
        HIP_TRY(ctx, launch_sample_small(ctx->d_primes, ctx->prm.seed, 5, ctr, (int)ctx->prm.noise, 0, ctx->d_gauss_cdt,
                                         ctx->gauss_cdt_n, all, 1, 0, 0, e.u(),
                                         nullptr, (int)ctx->log_n, ctx->stream));
        HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, e.u(), 0, (int)total, all, ctx->stream));
        HIP_TRY(ctx, launch_key_combine(ctx->d_primes, ctx->d_secret, target, e.u(), ctx->d_pmod, digit, (int)total,
                                        (int)ctx->L, (int)ctx->alpha, (int)j, (int)ctx->log_n, ctx->stream));
    }
    return HISA_OK;
}

// The key is registered only once every launch that builds it has been queued: a failure on the way (no memory for
// the temporary, a refused launch) frees the block and leaves no half-built key behind for later calls to trust.
static int gen_switch_key(hisa_ctx* ctx, u64 key_id, const u64* target) {
    const size_t words = (size_t)ctx->dnum * 2 * ctx->total * ctx->N;
    void* p = nullptr;
    HIP_TRY(ctx, hipMalloc(&p, words * sizeof(u64)));
    SwitchKey key{nullptr, (u64*)p};
    const int rc = fill_switch_key(ctx, key_id, target, key);
    if (rc != HISA_OK) {
        (void)hipStreamSynchronize(ctx->stream);   // nothing queued may still write to the block
        (void)hipFree(p);
        return rc;
    }
    key.blk = new DevBlock{p, words * sizeof(u64), 1};
    ctx->keys[key_id] = key;
    return HISA_OK;
}

extern "C" int hisa_keygen(hisa_ctx* ctx) {
    if (!ctx) return HISA_ERR_ARG;
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "keys cannot be generated during an analysis (no kernel runs)");
    if (ctx->keys.count(0)) return HISA_OK;
    Temp s2(ctx, (size_t)ctx->total * ctx->N * sizeof(u64));
    if (!s2.ok()) return HISA_ERR_OOM;
    HIP_TRY(ctx, launch_pointwise_square(ctx->d_primes, ctx->d_secret, s2.u(), (int)ctx->total, (int)ctx->log_n,
                                         ctx->stream));
    return gen_switch_key(ctx, 0, s2.u());
}

static u64 galois_of(const hisa_ctx* ctx, int32_t steps) {
    const u64 slots = ctx->N / 2, mask = 2 * (u64)ctx->N - 1;
    i64 r = (i64)steps % (i64)slots;
    if (r < 0) r += (i64)slots;
    u64 g = 1;
    for (i64 i = 0; i < r; i++) g = (g * 5) & mask;
    return r == 0 ? 0 : g;
}

extern "C" int hisa_galois_elt(hisa_ctx* ctx, int32_t left_steps, uint64_t* g) {
    if (!ctx || !g) return HISA_ERR_ARG;
    u64 v = galois_of(ctx, left_steps);
    *g = v ? v : 1;
    return HISA_OK;
}

extern "C" int hisa_gen_rot_keys(hisa_ctx* ctx, const int32_t* left_steps, size_t count) {
    if (!ctx || (!left_steps && count)) return fail(ctx, HISA_ERR_ARG, "null steps");
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "keys cannot be generated during an analysis (no kernel runs)");
    for (size_t i = 0; i < count; i++) {
        const u64 g = galois_of(ctx, left_steps[i]);
        if (g == 0 || ctx->keys.count(g)) continue;
        Temp tgt(ctx, (size_t)ctx->total * ctx->N * sizeof(u64));
        if (!tgt.ok()) return HISA_ERR_OOM;
        HIP_TRY(ctx, launch_automorph_ntt(ctx->d_secret, 0, tgt.u(), 0, g, (int)ctx->total, 1, (int)ctx->log_n, ctx->stream));
        TRY(gen_switch_key(ctx, g, tgt.u()));
    }
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// encode / decode / plaintexts
// ---------------------------------------------------------------------------
extern "C" int hisa_pt_from_coeffs(hisa_ctx* ctx, const int64_t* host_coeffs, double scale, uint32_t limbs, hisa_pt** out) {
    if (!ctx || !host_coeffs || !out || limbs < 1 || limbs > ctx->L) return fail(ctx, HISA_ERR_ARG, "bad argument");
    Temp co(ctx, ctx->N * sizeof(i64));
    if (!co.ok()) return HISA_ERR_OOM;
    HIP_TRY(ctx, hipMemcpyAsync(co.blk->ptr, host_coeffs, ctx->N * sizeof(i64), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));  // the host buffer may be reused by the caller
    TRY(alloc_pt(ctx, limbs, scale, out));
    HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co.as<i64>(), (*out)->data, (int)limbs, 1, (int)ctx->log_n, ctx->stream));
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, (*out)->data, 0, (int)limbs, identity_map((int)limbs), ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_encode(hisa_ctx* ctx, const double* re, const double* im, size_t count, double scale, uint32_t limbs,
                           hisa_pt** out) {
    if (!ctx || !out || (!re && count) || limbs < 1 || limbs > ctx->L || count > ctx->N / 2 || !(scale > 0))
        return fail(ctx, HISA_ERR_ARG, "bad argument");
    // coefficients must fit a signed 64-bit integer: |m_k| <= scale * max|z| * ~1
    Temp buf(ctx, (2 * count + 2) * sizeof(double));
    Temp co(ctx, ctx->N * sizeof(i64));
    if (!buf.ok() || !co.ok()) return HISA_ERR_OOM;
    double* d_re = buf.as<double>();
    double* d_im = im ? d_re + count : nullptr;
    if (count) HIP_TRY(ctx, hipMemcpyAsync(d_re, re, count * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    if (im && count) HIP_TRY(ctx, hipMemcpyAsync(d_im, im, count * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (count > 64) {   // the O(N log N) transform over the slot order; a handful of slots is cheaper summed directly
        Temp work(ctx, (ctx->N / 2) * 2 * sizeof(double));
        if (!work.ok()) return HISA_ERR_OOM;
        HIP_TRY(ctx, launch_encode_fft(ctx->d_cos, ctx->d_sin, ctx->d_pow5, d_re, d_im, nullptr, (int)count, 1,
                                       2.0 * scale / (double)ctx->N, work.blk->ptr, co.as<i64>(), (int)ctx->log_n, ctx->stream));
    } else {
        HIP_TRY(ctx, launch_encode(ctx->d_cos, ctx->d_sin, ctx->d_pow5, d_re, d_im, (int)count, 1, 2.0 * scale / (double)ctx->N,
                                   co.as<i64>(), (int)ctx->log_n, ctx->stream));
    }
    TRY(alloc_pt(ctx, limbs, scale, out));
    HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co.as<i64>(), (*out)->data, (int)limbs, 1, (int)ctx->log_n, ctx->stream));
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, (*out)->data, 0, (int)limbs, identity_map((int)limbs), ctx->stream));
    return HISA_OK;
}

// q_m^-1 mod q_i tables for the mixed-radix lift, built on first use
static int garner_tables(hisa_ctx* ctx, u64** inv, u64** inv_sh) {
    static const u64 KEY = 0;
    auto it = ctx->aux.find(KEY);
    if (it == ctx->aux.end()) {
        const size_t L = ctx->L;
        std::vector<u64> t(2 * L * L, 0);
        for (size_t m = 0; m < L; m++)
            for (size_t i = 0; i < L; i++) {
                if (i == m) continue;
                u64 v = hm::inv(ctx->mod[m] % ctx->mod[i], ctx->mod[i]);
                t[m * L + i] = v;
                t[L * L + m * L + i] = hm::shoup(v, ctx->mod[i]);
            }
        u64* d = nullptr;
        HIP_TRY(ctx, upload(&d, t));
        DevBlock* blk = new DevBlock{d, t.size() * sizeof(u64), 1};
        it = ctx->aux.emplace(KEY, SwitchKey{blk, d}).first;
    }
    *inv = it->second.data;
    *inv_sh = it->second.data + (size_t)ctx->L * ctx->L;
    return HISA_OK;
}

extern "C" int hisa_decode(hisa_ctx* ctx, const hisa_pt* pt, double* re, double* im, size_t count) {
    if (!ctx || !valid_pt(pt) || !re || count > ctx->N / 2) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const size_t n = ctx->N;
    Temp co(ctx, (size_t)pt->limbs * n * sizeof(u64));
    Temp m(ctx, n * sizeof(double));
    Temp z(ctx, (2 * count + 2) * sizeof(double));
    if (!co.ok() || !m.ok() || !z.ok()) return HISA_ERR_OOM;
    InttExtra ex = {};
    ex.in = pt->data;
    HIP_TRY(ctx, launch_intt(ctx->tabs, (int)ctx->log_n, co.u(), 0, (int)pt->limbs, identity_map((int)pt->limbs), &ex,
                             ctx->stream));
    u64 *ginv, *ginv_sh;
    TRY(garner_tables(ctx, &ginv, &ginv_sh));
    HIP_TRY(ctx, launch_crt_to_double(ctx->d_primes, co.u(), (int)pt->limbs, ginv, ginv_sh, (int)ctx->L, 1.0 / pt->scale,
                                      m.as<double>(), (int)ctx->log_n, ctx->stream));
    double* d_re = z.as<double>();
    double* d_im = d_re + count;
    if (count > 16) {
        Temp work(ctx, (n / 2) * 2 * sizeof(double));
        if (!work.ok()) return HISA_ERR_OOM;
        HIP_TRY(ctx, launch_decode_fft(ctx->d_cos, ctx->d_sin, ctx->d_pow5, m.as<double>(), (int)count, work.blk->ptr, d_re, d_im,
                                       (int)ctx->log_n, ctx->stream));
    } else {
        HIP_TRY(ctx, launch_decode(ctx->d_cos, ctx->d_sin, m.as<double>(), (int)count, d_re, d_im, (int)ctx->log_n, ctx->stream));
    }
    if (count) HIP_TRY(ctx, hipMemcpyAsync(re, d_re, count * sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    if (im && count) HIP_TRY(ctx, hipMemcpyAsync(im, d_im, count * sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_pt_export(hisa_ctx* ctx, const hisa_pt* pt, uint64_t* host) {
    if (!ctx || !valid_pt(pt) || !host) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const size_t words = (size_t)pt->limbs * ctx->N;
    Temp co(ctx, words * sizeof(u64));
    if (!co.ok()) return HISA_ERR_OOM;
    InttExtra ex = {};
    ex.in = pt->data;
    HIP_TRY(ctx, launch_intt(ctx->tabs, (int)ctx->log_n, co.u(), 0, (int)pt->limbs, identity_map((int)pt->limbs), &ex,
                             ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(host, co.u(), words * sizeof(u64), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_pt_info(const hisa_pt* pt, uint32_t* limbs, double* scale) {
    if (!valid_pt(pt)) return HISA_ERR_ARG;
    if (limbs) *limbs = pt->limbs;
    if (scale) *scale = pt->scale;
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// encryption profile
// ---------------------------------------------------------------------------
extern "C" int hisa_encrypt_batch(hisa_ctx* ctx, const hisa_pt* const* pts, size_t n, hisa_ct** out) {
    if (!ctx || !pts || !out || n == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    for (size_t i = 0; i < n; i++) {
        if (!valid_pt(pts[i])) return fail(ctx, HISA_ERR_ARG, "entry %zu is not a plaintext", i);
        if (pts[i]->limbs != pts[0]->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "plaintexts differ in level");
    }
    const uint32_t l = pts[0]->limbs;
    const size_t nn = ctx->N, lw = (size_t)l * nn;
    TRY(alloc_ct_batch(ctx, n, 2, l, pts[0]->scale, out));
    for (size_t i = 0; i < n; i++) out[i]->scale = pts[i]->scale;
    u64* ct = out[0]->data;
    Temp e(ctx, n * lw * sizeof(u64));
    Temp ptbuf(ctx, n * lw * sizeof(u64));
    if (!e.ok() || !ptbuf.ok()) return HISA_ERR_OOM;
    PolyMap lm = identity_map((int)l);
    // c1 = a: uniform in coefficient form, then NTT.  Treat (ciphertext, poly 1) as batch entries of stride 2*l*N.
    HIP_TRY(ctx, launch_sample_uniform(ctx->d_primes, ctx->prm.seed, 2, ctx->enc_counter, lm, (int)(n * l), 2 * lw, 1,
                                       ct + lw, (int)ctx->log_n, ctx->stream));
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, ct + lw, 2 * lw, (int)(n * l), lm, ctx->stream));
    HIP_TRY(ctx, launch_sample_small(ctx->d_primes, ctx->prm.seed, 3, ctx->enc_counter, (int)ctx->prm.noise, 0, ctx->d_gauss_cdt,
                                     ctx->gauss_cdt_n, lm, (int)n,
                                     lw, 1, e.u(), nullptr, (int)ctx->log_n, ctx->stream));
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, e.u(), lw, (int)(n * l), lm, ctx->stream));
    const u64* pt_base = pts[0]->data;
    u64 pt_bs = 0;
    if (n > 1) {
        for (size_t i = 0; i < n; i++)
            HIP_TRY(ctx, hipMemcpyAsync(ptbuf.u() + i * lw, pts[i]->data, lw * sizeof(u64), hipMemcpyDeviceToDevice,
                                        ctx->stream));
        pt_base = ptbuf.u();
        pt_bs = lw;
    }
    HIP_TRY(ctx, launch_encrypt_combine(ctx->d_primes, ctx->d_secret, pt_base, e.u(), ct, (int)l, n, pt_bs, (int)ctx->log_n,
                                        ctx->stream));
    ctx->enc_counter += n;
    return HISA_OK;
}

extern "C" int hisa_encrypt(hisa_ctx* ctx, const hisa_pt* pt, hisa_ct** out) { return hisa_encrypt_batch(ctx, &pt, 1, out); }

extern "C" int hisa_set_enc_counter(hisa_ctx* ctx, uint64_t counter) {
    if (!ctx) return HISA_ERR_ARG;
    ctx->enc_counter = counter;
    return HISA_OK;
}

extern "C" int hisa_decrypt(hisa_ctx* ctx, const hisa_ct* ct, hisa_pt** out) {
    if (!ctx || !valid_ct(ct) || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_pt(ctx, ct->limbs, ct->scale, out));
    HIP_TRY(ctx, launch_decrypt(ctx->d_primes, ctx->d_secret, ct->data, (*out)->data, (int)ct->limbs, (int)ct->polys,
                                (int)ctx->log_n, ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_copy(hisa_ctx* ctx, const hisa_ct* ct, hisa_ct** out) {
    if (!ctx || !valid_ct(ct) || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_ct_batch(ctx, 1, ct->polys, ct->limbs, ct->scale, out));
    HIP_TRY(ctx, hipMemcpyAsync((*out)->data, ct->data, ct_words(ctx, ct->polys, ct->limbs) * sizeof(u64),
                                hipMemcpyDeviceToDevice, ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_free(hisa_ctx* ctx, void* handle) {
    if (!handle) return HISA_OK;
    if (!ctx) return HISA_ERR_ARG;
    uint32_t magic = *(uint32_t*)handle;
    if (magic == HISA_MAGIC_CT) {
        hisa_ct* c = (hisa_ct*)handle;
        dev_release(ctx, c->blk);
        c->magic = 0;
        delete c;
    } else if (magic == HISA_MAGIC_PT) {
        hisa_pt* p = (hisa_pt*)handle;
        dev_release(ctx, p->blk);
        p->magic = 0;
        delete p;
    } else {
        return fail(ctx, HISA_ERR_ARG, "not a live handle");
    }
    return HISA_OK;
}

// swap the storage of an in-place result into the caller's handle
static void adopt(hisa_ctx* ctx, hisa_ct* dst, hisa_ct* src) {
    dev_release(ctx, dst->blk);
    dst->blk = src->blk; dst->data = src->data; dst->polys = src->polys; dst->limbs = src->limbs; dst->scale = src->scale;
    src->magic = 0;
    delete src;
}

// ---------------------------------------------------------------------------
// add / sub
// ---------------------------------------------------------------------------
static bool same_scale(double a, double b) { return fabs(a - b) <= ldexp(fmax(fabs(a), fabs(b)), -30); }

static int addsub_into(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, int op, u64* dst) {
    HIP_TRY(ctx, launch_addsub(ctx->d_primes, a->data, b->data, dst, op, (int)a->limbs, (int)a->polys, (int)b->polys, 1, 0,
                               0, 0, (int)ctx->log_n, ctx->stream));
    return HISA_OK;
}

static int addsub_check(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b) {
    if (!ctx || !valid_ct(a) || !valid_ct(b)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (a->limbs != b->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "levels %u and %u", a->limbs, b->limbs);
    if (!same_scale(a->scale, b->scale)) return fail(ctx, HISA_ERR_SCALE_MISMATCH, "scales %g and %g", a->scale, b->scale);
    return HISA_OK;
}

static int addsub(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, int op, hisa_ct** out) {
    TRY(addsub_check(ctx, a, b));
    if (!out) return fail(ctx, HISA_ERR_ARG, "null out");
    if (a->polys < b->polys) {
        if (op == OP_SUB) return fail(ctx, HISA_ERR_SIZE, "subtrahend has more polynomials");
        std::swap(a, b);
    }
    TRY(alloc_ct_batch(ctx, 1, a->polys, a->limbs, a->scale, out));
    return addsub_into(ctx, a, b, op, (*out)->data);
}

static int addsub_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b, int op) {
    TRY(addsub_check(ctx, a, b));
    if (a->polys < b->polys) return fail(ctx, HISA_ERR_SIZE, "right operand has more polynomials");
    return addsub_into(ctx, a, b, op, a->data);
}

extern "C" int hisa_add(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out) { return addsub(ctx, a, b, OP_ADD, out); }
extern "C" int hisa_sub(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out) { return addsub(ctx, a, b, OP_SUB, out); }
extern "C" int hisa_add_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b) { return addsub_assign(ctx, a, b, OP_ADD); }
extern "C" int hisa_sub_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b) { return addsub_assign(ctx, a, b, OP_SUB); }

static int addsub_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, int op, u64* dst) {
    // the plaintext is a one-polynomial operand: polys_b = 1
    HIP_TRY(ctx, launch_addsub(ctx->d_primes, a->data, p->data, dst, op, (int)a->limbs, (int)a->polys, 1, 1, 0, 0, 0,
                               (int)ctx->log_n, ctx->stream));
    return HISA_OK;
}

static int plain_check(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, bool need_scale) {
    if (!ctx || !valid_ct(a) || !valid_pt(p)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (a->limbs != p->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "levels %u and %u", a->limbs, p->limbs);
    if (need_scale && !same_scale(a->scale, p->scale))
        return fail(ctx, HISA_ERR_SCALE_MISMATCH, "scales %g and %g", a->scale, p->scale);
    return HISA_OK;
}

static int addsub_plain_new(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, int op, hisa_ct** out) {
    TRY(plain_check(ctx, a, p, true));
    if (!out) return fail(ctx, HISA_ERR_ARG, "null out");
    TRY(alloc_ct_batch(ctx, 1, a->polys, a->limbs, a->scale, out));
    return addsub_plain(ctx, a, p, op, (*out)->data);
}

extern "C" int hisa_add_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out) { return addsub_plain_new(ctx, a, p, OP_ADD, out); }
extern "C" int hisa_sub_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out) { return addsub_plain_new(ctx, a, p, OP_SUB, out); }
extern "C" int hisa_add_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p) {
    TRY(plain_check(ctx, a, p, true));
    return addsub_plain(ctx, a, p, OP_ADD, a->data);
}
extern "C" int hisa_sub_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p) {
    TRY(plain_check(ctx, a, p, true));
    return addsub_plain(ctx, a, p, OP_SUB, a->data);
}

static int addsub_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, int op, u64* dst) {
    u64 consts[HISA_MAX_PRIMES];
    const double v = x * a->scale;
    if (!isfinite(v)) return fail(ctx, HISA_ERR_ARG, "scalar times scale is not finite");
    for (uint32_t i = 0; i < a->limbs; i++) consts[i] = hm::double_to_residue(v, ctx->mod[i]);
    HIP_TRY(ctx, launch_add_const(ctx->d_primes, a->data, dst, consts, op, (int)a->limbs, (int)a->polys, (int)ctx->log_n,
                                  ctx->stream));
    return HISA_OK;
}

static int addsub_scalar_new(hisa_ctx* ctx, const hisa_ct* a, double x, int op, hisa_ct** out) {
    if (!ctx || !valid_ct(a) || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_ct_batch(ctx, 1, a->polys, a->limbs, a->scale, out));
    return addsub_scalar(ctx, a, x, op, (*out)->data);
}

extern "C" int hisa_add_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, hisa_ct** out) { return addsub_scalar_new(ctx, a, x, OP_ADD, out); }
extern "C" int hisa_sub_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, hisa_ct** out) { return addsub_scalar_new(ctx, a, x, OP_SUB, out); }
extern "C" int hisa_add_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x) {
    if (!ctx || !valid_ct(a)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    return addsub_scalar(ctx, a, x, OP_ADD, a->data);
}
extern "C" int hisa_sub_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x) {
    if (!ctx || !valid_ct(a)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    return addsub_scalar(ctx, a, x, OP_SUB, a->data);
}

extern "C" int hisa_add_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_ct* const* b, size_t n, hisa_ct** out) {
    if (!ctx || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, a, n, 0));
    TRY(check_batch_shape(ctx, b, n, a[0]->polys));
    for (size_t i = 0; i < n; i++) TRY(addsub_check(ctx, a[i], b[i]));
    BatchIn ia, ib;
    TRY(gather_batch(ctx, a, n, &ia));
    int rc = gather_batch(ctx, b, n, &ib);
    if (rc == HISA_OK) rc = alloc_ct_batch(ctx, n, a[0]->polys, a[0]->limbs, a[0]->scale, out);
    if (rc == HISA_OK) {
        for (size_t i = 0; i < n; i++) out[i]->scale = a[i]->scale;
        hipError_t e = launch_addsub(ctx->d_primes, ia.base, ib.base, out[0]->data, OP_ADD, (int)a[0]->limbs, (int)a[0]->polys,
                                     (int)a[0]->polys, n, ia.stride, ib.stride, ia.stride, (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "add batch: %s", hipGetErrorString(e));
    }
    dev_release(ctx, ia.tmp);
    dev_release(ctx, ib.tmp);
    return rc;
}

// ---------------------------------------------------------------------------
// multiply
// ---------------------------------------------------------------------------
extern "C" int hisa_mul_plain_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_pt* p, size_t n, hisa_ct** out) {
    if (!ctx || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, a, n, 0));
    TRY(plain_check(ctx, a[0], p, false));
    BatchIn ia;
    TRY(gather_batch(ctx, a, n, &ia));
    int rc = alloc_ct_batch(ctx, n, a[0]->polys, a[0]->limbs, a[0]->scale * p->scale, out);
    if (rc == HISA_OK) {
        for (size_t i = 0; i < n; i++) out[i]->scale = a[i]->scale * p->scale;
        hipError_t e = launch_mul_plain(ctx->d_primes, ia.base, p->data, out[0]->data, (int)a[0]->limbs, (int)a[0]->polys, n,
                                        ia.stride, ia.stride, (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "mul_plain: %s", hipGetErrorString(e));
    }
    dev_release(ctx, ia.tmp);
    return rc;
}

extern "C" int hisa_mul_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out) {
    return hisa_mul_plain_batch(ctx, &a, p, 1, out);
}

extern "C" int hisa_mul_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p) {
    TRY(plain_check(ctx, a, p, false));
    HIP_TRY(ctx, launch_mul_plain(ctx->d_primes, a->data, p->data, a->data, (int)a->limbs, (int)a->polys, 1, 0, 0,
                                  (int)ctx->log_n, ctx->stream));
    a->scale *= p->scale;
    return HISA_OK;
}

static int mul_scalar_into(hisa_ctx* ctx, const hisa_ct* a, double x, double x_scale, u64* dst) {
    u64 consts[2 * HISA_MAX_PRIMES];
    const double v = x * x_scale;
    if (!isfinite(v)) return fail(ctx, HISA_ERR_ARG, "scalar times scale is not finite");
    for (uint32_t i = 0; i < a->limbs; i++) {
        consts[i] = hm::double_to_residue(v, ctx->mod[i]);
        consts[a->limbs + i] = hm::shoup(consts[i], ctx->mod[i]);
    }
    HIP_TRY(ctx, launch_mul_const(ctx->d_primes, a->data, dst, consts, (int)a->limbs, (int)a->polys, (int)ctx->log_n,
                                  ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_mul_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, double x_scale, hisa_ct** out) {
    if (!ctx || !valid_ct(a) || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_ct_batch(ctx, 1, a->polys, a->limbs, a->scale * x_scale, out));
    return mul_scalar_into(ctx, a, x, x_scale, (*out)->data);
}

extern "C" int hisa_mul_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x, double x_scale) {
    if (!ctx || !valid_ct(a)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(mul_scalar_into(ctx, a, x, x_scale, a->data));
    a->scale *= x_scale;
    return HISA_OK;
}

extern "C" int hisa_mul_no_relin_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_ct* const* b, size_t n,
                                       hisa_ct** out) {
    if (!ctx || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, a, n, 2));
    TRY(check_batch_shape(ctx, b, n, 2));
    if (a[0]->limbs != b[0]->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "levels %u and %u", a[0]->limbs, b[0]->limbs);
    BatchIn ia, ib;
    TRY(gather_batch(ctx, a, n, &ia));
    int rc = gather_batch(ctx, b, n, &ib);
    if (rc == HISA_OK) rc = alloc_ct_batch(ctx, n, 3, a[0]->limbs, 0.0, out);
    if (rc == HISA_OK) {
        for (size_t i = 0; i < n; i++) out[i]->scale = a[i]->scale * b[i]->scale;
        hipError_t e = launch_mul_no_relin(ctx->d_primes, ia.base, ib.base, out[0]->data, (int)a[0]->limbs, n, ia.stride,
                                           ib.stride, ct_words(ctx, 3, a[0]->limbs), (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "mul_no_relin: %s", hipGetErrorString(e));
    }
    dev_release(ctx, ia.tmp);
    dev_release(ctx, ib.tmp);
    return rc;
}

extern "C" int hisa_mul_no_relin(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out) {
    return hisa_mul_no_relin_batch(ctx, &a, &b, 1, out);
}

// ---------------------------------------------------------------------------
// hybrid key switching
// ---------------------------------------------------------------------------
// Per-level factors that close the inverse transform of the polynomial to be
// switched: N^-1 * (D_j / q_i)^-1 mod q_i for limb i in digit j.
struct LevelPost {
    u64* d;  // [l] values then [l] Shoup companions
};

static int level_post(hisa_ctx* ctx, int l, u64** post, u64** post_sh) {
    const u64 KEY = 16 + (u64)l;
    auto it = ctx->aux.find(KEY);
    if (it == ctx->aux.end()) {
        std::vector<u64> t(2 * (size_t)l);
        const int digits = (l + (int)ctx->alpha - 1) / (int)ctx->alpha;
        for (int j = 0; j < digits; j++) {
            const int lo = j * (int)ctx->alpha, hi = std::min(lo + (int)ctx->alpha, l);
            ConvTable* tab;
            TRY(modup_table(ctx, j, hi - lo, &tab));
            for (int i = lo; i < hi; i++) {
                const u64 q = ctx->mod[i];
                t[i] = hm::mul(ctx->pc[i].n_inv, tab->inv_hat[i - lo], q);
                t[l + i] = hm::shoup(t[i], q);
            }
        }
        u64* d = nullptr;
        HIP_TRY(ctx, upload(&d, t));
        it = ctx->aux.emplace(KEY, SwitchKey{new DevBlock{d, t.size() * sizeof(u64), 1}, d}).first;
    }
    *post = it->second.data;
    *post_sh = it->second.data + l;
    return HISA_OK;
}

static int moddown_post(hisa_ctx* ctx, u64** post, u64** post_sh) {
    const u64 KEY = 1;
    auto it = ctx->aux.find(KEY);
    if (it == ctx->aux.end()) {
        // laid out for a PolyMap of period l + K is not possible (l varies), so the table is indexed by
        // special-prime number and the caller offsets the pointer by -l
        std::vector<u64> t(2 * (size_t)ctx->K);
        for (uint32_t m = 0; m < ctx->K; m++) {
            const u64 q = ctx->mod[ctx->L + m];
            t[m] = hm::mul(ctx->pc[ctx->L + m].n_inv, ctx->moddown_tab->inv_hat[m], q);
            t[ctx->K + m] = hm::shoup(t[m], q);
        }
        u64* d = nullptr;
        HIP_TRY(ctx, upload(&d, t));
        it = ctx->aux.emplace(KEY, SwitchKey{new DevBlock{d, t.size() * sizeof(u64), 1}, d}).first;
    }
    *post = it->second.data;
    *post_sh = it->second.data + ctx->K;
    return HISA_OK;
}

// Key switch of B polynomials d[b] (NTT form, l limbs, at d + b*d_bs) under `key`;
// out[b] = (ks0 + add0, ks1 + add1) with the optional addends taken from
// add + b*add_bs (add_polys polynomials of l limbs, read through sigma_g when add_galois != 0).
static int key_switch_core(hisa_ctx* ctx, const u64* d, u64 d_bs, size_t B, int l, const SwitchKey& key, const u64* add,
                           u64 add_bs, int add_polys, u64 add_galois, u64* out) {
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total;
    const int ext_limbs = l + K;
    const int digits = (l + alpha - 1) / alpha;
    const int log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;

    Temp y(ctx, B * l * n * sizeof(u64));
    Temp ext(ctx, B * (size_t)digits * ext_limbs * n * sizeof(u64));
    Temp acc(ctx, B * 2 * (size_t)ext_limbs * n * sizeof(u64));
    Temp conv(ctx, B * 2 * (size_t)l * n * sizeof(u64));
    if (!y.ok() || !ext.ok() || !acc.ok() || !conv.ok()) return HISA_ERR_OOM;
    const u64 ext_bs = (u64)digits * ext_limbs * n;

    // 1. coefficient form, each limb pre-multiplied by (D_j/q_i)^-1
    u64 *post, *post_sh;
    TRY(level_post(ctx, l, &post, &post_sh));
    InttExtra ex = {};
    ex.in = d; ex.in_batch_stride = d_bs; ex.post = post; ex.post_sh = post_sh;
    HIP_TRY(ctx, launch_intt(ctx->tabs, log_n, y.u(), (u64)l * n, (int)(B * l), identity_map(l), &ex, st));

    // 2.-3. per digit: convert to every other prime, transform; own primes keep the input's NTT form
    for (int j = 0; j < digits; j++) {
        const int lo = j * alpha, hi = std::min(lo + alpha, l);
        ConvTable* tab;
        TRY(modup_table(ctx, j, hi - lo, &tab));
        ConvArgs ca = {};
        ca.y = y.u(); ca.y_bs = (u64)l * n; ca.src_pos0 = lo; ca.src_prime0 = lo; ca.a = hi - lo;
        ca.hat = tab->d_hat; ca.dmod = tab->d_dmod; ca.total = total;
        ca.out = ext.u() + (size_t)j * ext_limbs * n; ca.out_bs = ext_bs;
        PolyMap pm = {};
        pm.period = ext_limbs;
        int nt = 0;
        for (int x = 0; x < ext_limbs; x++) {
            const int prime = x < l ? x : L + (x - l);
            const bool own = x >= lo && x < hi;
            pm.prime_of[x] = own ? (int16_t)-1 : (int16_t)prime;
            if (!own) { ca.tgt_pos[nt] = (int16_t)x; ca.tgt_prime[nt] = (int16_t)prime; nt++; }
        }
        ca.n_targets = nt;
        HIP_TRY(ctx, launch_base_conv(ctx->d_primes, ca, B, log_n, st));
        HIP_TRY(ctx, launch_copy_limbs(d + (size_t)lo * n, d_bs, ext.u() + ((size_t)j * ext_limbs + lo) * n, ext_bs, hi - lo, B,
                                       log_n, st));
        // batch entries of this digit are ext_bs apart
        HIP_TRY(ctx, launch_ntt(ctx->tabs, log_n, ext.u() + (size_t)j * ext_limbs * n, ext_bs, (int)(B * ext_limbs), pm, st));
    }

    // 4. inner product with the key
    HIP_TRY(ctx, launch_inner_product(ctx->d_primes, ext.u(), ext_bs, digits, l, K, L, key.data, total, acc.u(),
                                      (u64)2 * ext_limbs * n, B, log_n, st));

    // 5. mod-down: special limbs to coefficient form (pre-multiplied by (P/p_m)^-1), convert, transform, combine
    u64 *mpost, *mpost_sh;
    TRY(moddown_post(ctx, &mpost, &mpost_sh));
    {
        PolyMap pm = {};
        pm.period = ext_limbs;
        for (int x = 0; x < ext_limbs; x++) pm.prime_of[x] = x < l ? (int16_t)-1 : (int16_t)(L + x - l);
        InttExtra ex2 = {};
        ex2.post = mpost - l; ex2.post_sh = mpost_sh - l;  // entry x >= l reads post[x - l]
        HIP_TRY(ctx, launch_intt(ctx->tabs, log_n, acc.u(), (u64)ext_limbs * n, (int)(B * 2 * ext_limbs), pm, &ex2, st));
        ConvArgs ca = {};
        ca.y = acc.u(); ca.y_bs = (u64)ext_limbs * n; ca.src_pos0 = l; ca.src_prime0 = L; ca.a = K;
        ca.hat = ctx->moddown_tab->d_hat; ca.dmod = ctx->moddown_tab->d_dmod; ca.total = total;
        ca.out = conv.u(); ca.out_bs = (u64)l * n; ca.n_targets = l;
        for (int i = 0; i < l; i++) { ca.tgt_pos[i] = (int16_t)i; ca.tgt_prime[i] = (int16_t)i; }
        HIP_TRY(ctx, launch_base_conv(ctx->d_primes, ca, B * 2, log_n, st));
        HIP_TRY(ctx, launch_ntt(ctx->tabs, log_n, conv.u(), (u64)l * n, (int)(B * 2 * l), identity_map(l), st));
    }
    HIP_TRY(ctx, launch_moddown_final(ctx->d_primes, acc.u(), (u64)2 * ext_limbs * n, conv.u(), (u64)2 * l * n, ctx->d_pinv,
                                      ctx->d_pinv_sh, add, add_bs, add_polys, add_galois, out, (u64)2 * l * n, l, K, B, log_n,
                                      st));
    return HISA_OK;
}

// (D_j/q_i)^-1 of every limb at level l (and (P/p_m)^-1 of the special primes) as centred doubles, device resident
static int fp_post_tables(hisa_ctx* ctx, int l, double** post_q, double** post_p, bool lookup_only) {
    const u64 KEY = 4096 + (u64)l;
    auto it = ctx->aux.find(KEY);
    if (it == ctx->aux.end() && lookup_only) return fail(ctx, HISA_ERR_ARG, "no conversion tables for level %d", l);
    if (it == ctx->aux.end()) {
        std::vector<double> t((size_t)l + ctx->K);
        const int digits = (l + (int)ctx->alpha - 1) / (int)ctx->alpha;
        for (int j = 0; j < digits; j++) {
            const int lo = j * (int)ctx->alpha, hi = std::min(lo + (int)ctx->alpha, l);
            ConvTable* tab;
            TRY(modup_table(ctx, j, hi - lo, &tab));
            for (int i = lo; i < hi; i++) t[i] = centred_double(tab->inv_hat[i - lo], ctx->mod[i]);
        }
        for (uint32_t m = 0; m < ctx->K; m++) t[l + m] = centred_double(ctx->moddown_tab->inv_hat[m], ctx->mod[ctx->L + m]);
        double* d = nullptr;
        HIP_TRY(ctx, upload(&d, t));
        it = ctx->aux.emplace(KEY, SwitchKey{new DevBlock{d, t.size() * sizeof(double), 1}, (u64*)d}).first;
    }
    *post_q = (double*)it->second.data;
    *post_p = (double*)it->second.data + l;
    return HISA_OK;
}

// Hybrid key switch of B polynomials with the fused fp64 kernels (all primes below 2^50):
//   A  inverse transform of d (read through sigma_g if galois != 0) times (D_j/q_i)^-1  -> y, centred doubles
//   B  per digit: base conversion of y to every other prime fused into the forward transform -> ext
//   IP inner product with the key; a digit's own limbs are read from d itself             -> acc (l + K limbs, b|a)
//   C  inverse transform of the K special limbs of acc times (P/p_m)^-1                    -> y2
//   D  base conversion of y2 to q_i fused into the forward transform, then (acc - conv) P^-1 + addend -> out
// A and B (the decomposition and ModUp) are one function, IP, C and D another, so that several rotations of the same
// ciphertexts can share the first: the conversion works coefficient by coefficient on centred values, so it commutes
// with the automorphism, which then becomes a gather on the extended digits inside IP.
struct FpExt {
    Temp y, ext;       // pooled buffers, or empty when the caller brought a workspace
    double* yp;        // [B][l][N] centred doubles
    double* extp;      // [B][digits][l + K][N], lazily reduced doubles
    int l, digits, ext_limbs;
    u64 ext_bs;
    static size_t y_bytes(const hisa_ctx* ctx, size_t B, int l) { return B * (size_t)l * ctx->N * sizeof(double); }
    static size_t ext_bytes(const hisa_ctx* ctx, size_t B, int l, int K, int alpha) {
        return B * (size_t)((l + alpha - 1) / alpha) * (size_t)(l + K) * ctx->N * sizeof(u64);
    }
    FpExt(hisa_ctx* ctx, size_t B, int l_, int K, int alpha)
        : y(ctx, y_bytes(ctx, B, l_)), ext(ctx, ext_bytes(ctx, B, l_, K, alpha)),
          yp(y.ok() ? y.as<double>() : nullptr), extp(ext.ok() ? ext.as<double>() : nullptr),
          l(l_), digits((l_ + alpha - 1) / alpha), ext_limbs(l_ + K), ext_bs((u64)digits * ext_limbs * ctx->N) {}
    // the same two buffers inside memory the caller owns: nothing is allocated
    FpExt(hisa_ctx* ctx, int l_, int K, int alpha, double* y_ws, double* ext_ws)
        : y(ctx, Temp::None()), ext(ctx, Temp::None()), yp(y_ws), extp(ext_ws),
          l(l_), digits((l_ + alpha - 1) / alpha), ext_limbs(l_ + K), ext_bs((u64)digits * ext_limbs * ctx->N) {}
    bool ok() const { return yp && extp; }
};

static FpArgs fp_base(hisa_ctx* ctx) {
    FpArgs base = {};
    base.fprimes = ctx->tabs.fprimes; base.ftw = ctx->tabs.ftw; base.utw = ctx->tabs.utw; base.vtw = ctx->tabs.vtw;
    base.scratch = ctx->d_fp_scratch; base.scratch_polys = ctx->fp_scratch_polys;
    return base;
}

static int key_switch_modup_fp(hisa_ctx* ctx, const u64* d, u64 d_bs, u64 galois, size_t B, FpExt& x, bool no_alloc = false) {
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, l = x.l;
    const int log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;
    double *post_q, *post_p;
    TRY(fp_post_tables(ctx, l, &post_q, &post_p, no_alloc));
    FpArgs base = fp_base(ctx);
    if (no_alloc) { base.scratch = nullptr; base.scratch_polys = 0; base.no_pair = 1; }
    {   // A
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l;
        for (int i = 0; i < l; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.in = d; a.in_bs = d_bs; a.galois = galois; a.post = post_q;
        a.yout = x.yp; a.yout_bs = (u64)l * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_TO_Y, log_n, a, tk, B, st));
    }
    // B.  One launch per digit, or one for all digits (single target limbs) where that takes fewer rounds of
    // workgroups: small batches, whose per-digit launches would each run one sparse round after the other
    size_t all_targets = 0;
    double separate = 0.0;
    for (int j = 0; j < x.digits; j++) {
        const int own = std::min(j * alpha + alpha, l) - j * alpha;
        all_targets += (size_t)(x.ext_limbs - own);
        separate += fp_conversion_cost(log_n, own, x.ext_limbs - own, B, nullptr);
    }
    const u64 resident = fp_resident_workgroups(log_n);
    const bool one_launch = x.digits > 1 && x.digits <= FP_MAX_DIGITS && all_targets <= HISA_MAX_PRIMES &&
                            (double)((B * all_targets + resident - 1) / resident) <= separate;
    FpArgs a = base;
    FpTask tk = {};
    int cnt = 0;
    a.y = x.yp; a.y_bs = (u64)l * n; a.total = total;
    a.out = (u64*)x.extp; a.out_bs = x.ext_bs;
    for (int j = 0; j < x.digits; j++) {
        const int lo = j * alpha, hi = std::min(lo + alpha, l);
        ConvTable* tab;
        if (no_alloc) {   // built with the level's tables when the context was made
            auto it = ctx->modup_tabs.find(std::make_pair(j, hi - lo));
            if (it == ctx->modup_tabs.end()) return fail(ctx, HISA_ERR_ARG, "no conversion table for digit %d of %d limbs", j, hi - lo);
            tab = &it->second;
        } else {
            TRY(modup_table(ctx, j, hi - lo, &tab));
        }
        const int slot = one_launch ? j : 0;
        a.dg[slot].hat = tab->d_hat_f; a.dg[slot].y_pos0 = lo; a.dg[slot].conv_a = hi - lo;
        if (!one_launch) cnt = 0;
        for (int e = 0; e < x.ext_limbs; e++) {
            if (e >= lo && e < hi) continue;
            tk.pos[cnt] = (int16_t)(j * x.ext_limbs + e);
            tk.prime[cnt] = (int16_t)(e < l ? e : L + (e - l));
            tk.digit[cnt] = (int8_t)slot;
            cnt++;
        }
        if (!one_launch || j == x.digits - 1) {
            tk.period = cnt;
            a.n_digits = one_launch ? x.digits : 1;
            HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV, log_n, a, tk, B, st));
        }
    }
    return HISA_OK;
}

// IP, C, D.  `galois` is applied to the own-digit limbs read from d, to the addend, and (gather_ext) to the digits.
// C, D: acc [B][2][l + K][N] (NTT form) -> out[B][2][l][N] = ModDown(acc) (+ addend, gathered through add_galois if set)
int moddown_add_fp(hisa_ctx* ctx, const u64* acc, size_t B, int l, const u64* add, u64 add_bs, int add_polys, u64 add_galois,
                   u64* out, double* y2_ws) {
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, total = (int)ctx->total, ext_limbs = l + K, log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;
    // y2_ws: the caller's memory for the conversion input ([B][2][K][N] doubles); then nothing is allocated here
    const bool no_alloc = y2_ws != nullptr;
    Temp y2_t(ctx, B * 2 * (size_t)K * n * sizeof(double), !no_alloc);
    if (!no_alloc && !y2_t.ok()) return HISA_ERR_OOM;
    double* y2 = no_alloc ? y2_ws : y2_t.as<double>();
    double *post_q, *post_p;
    TRY(fp_post_tables(ctx, l, &post_q, &post_p, no_alloc));
    FpArgs base = fp_base(ctx);
    if (no_alloc) { base.scratch = nullptr; base.scratch_polys = 0; base.no_pair = 1; }
    {   // C: batch entries are (ciphertext, b|a) pairs
        FpArgs a = base;
        FpTask tk = {};
        tk.period = K;
        for (int m = 0; m < K; m++) { tk.pos[m] = (int16_t)m; tk.prime[m] = (int16_t)(L + m); }
        a.in = acc; a.in_bs = (u64)ext_limbs * n; a.in_pos_shift = l; a.post = post_p;
        a.yout = y2; a.yout_bs = (u64)K * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_TO_Y, log_n, a, tk, B * 2, st));
    }
    {   // D
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l;
        for (int i = 0; i < l; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.y = y2; a.y_bs = (u64)K * n; a.y_pos0 = 0; a.conv_a = K; a.total = total; a.hat = ctx->moddown_tab->d_hat_f;
        a.acc = acc; a.acc_bs = (u64)ext_limbs * n; a.acc_pos_shift = 0; a.pinv_tab = ctx->d_pinv_f;
        a.add = add; a.add_bs = add_bs; a.add_ps = (u64)l * n; a.add_div = 2; a.add_polys = add_polys; a.add_galois = add_galois;
        a.out = out; a.out_bs = (u64)l * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV_FINAL, log_n, a, tk, B * 2, st));
    }
    return HISA_OK;
}

// Tables of the combined division at level l: sources q_{l-1}, p_0 .. p_{K-1} (conversion table; (D/s_m)^-1 as centred
// doubles, D = q_{l-1} P) and D^-1 mod q_i as centred doubles indexed by prime
static int moddown_rescale_tables(hisa_ctx* ctx, int l, ConvTable** tab, double** post, double** dinv) {
    const auto key = std::make_pair(-l, (int)ctx->K + 1);
    auto it = ctx->modup_tabs.find(key);
    if (it == ctx->modup_tabs.end()) {
        std::vector<int> src(1, l - 1);
        for (uint32_t m = 0; m < ctx->K; m++) src.push_back((int)(ctx->L + m));
        ConvTable t = {};
        TRY(make_conv_table(ctx, src, &t));
        it = ctx->modup_tabs.emplace(key, t).first;
    }
    *tab = &it->second;
    const u64 KEY = 12288 + (u64)l;     // (8192 + l: the constants of the plain rescale)
    auto ia = ctx->aux.find(KEY);
    if (ia == ctx->aux.end()) {
        const ConvTable& t = it->second;
        std::vector<double> v((size_t)t.a + ctx->total, 0.0);
        for (int m = 0; m < t.a; m++) v[m] = centred_double(t.inv_hat[m], ctx->mod[t.src[m]]);
        for (int i = 0; i < l - 1; i++) {
            const u64 q = ctx->mod[i];
            u64 d = 1 % q;
            for (int m = 0; m < t.a; m++) d = hm::mul(d, ctx->mod[t.src[m]] % q, q);
            v[(size_t)t.a + i] = centred_double(hm::inv(d, q), q);
        }
        double* dev = nullptr;
        HIP_TRY(ctx, upload(&dev, v));
        ia = ctx->aux.emplace(KEY, SwitchKey{new DevBlock{dev, v.size() * sizeof(double), 1}, (u64*)dev}).first;
    }
    *post = (double*)ia->second.data;
    *dinv = (double*)ia->second.data + it->second.a;
    return HISA_OK;
}

int moddown_rescale_fp(hisa_ctx* ctx, u64* acc, size_t B, int l, const u64* add, u64 add_bs, int add_polys, u64* out) {
    if (!fused_key_switch_available(ctx)) return fail(ctx, HISA_ERR_ARG, "no fused key-switch path for these parameters");
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "no level to rescale into");
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, total = (int)ctx->total, ext_limbs = l + K, log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;
    ConvTable* tab;
    double *post, *dinv;
    TRY(moddown_rescale_tables(ctx, l, &tab, &post, &dinv));
    Temp y2(ctx, B * 2 * (size_t)(K + 1) * n * sizeof(double));
    if (!y2.ok()) return HISA_ERR_OOM;
    if (add)
        HIP_TRY(ctx, launch_fold_addend(ctx->d_primes, acc, (u64)ext_limbs * n, add, add_bs, (u64)l * n, add_polys, ctx->d_pmod, B, l,
                                        log_n, st));
    const FpArgs base = fp_base(ctx);
    {   // the limb of q_{l-1} and the special limbs to coefficient form, times (D/s_m)^-1
        FpArgs a = base;
        FpTask tk = {};
        tk.period = K + 1;
        for (int m = 0; m <= K; m++) { tk.pos[m] = (int16_t)m; tk.prime[m] = (int16_t)(m == 0 ? l - 1 : L + m - 1); }
        a.in = acc; a.in_bs = (u64)ext_limbs * n; a.in_pos_shift = l - 1; a.post = post;
        a.yout = y2.as<double>(); a.yout_bs = (u64)(K + 1) * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_TO_Y, log_n, a, tk, B * 2, st));
    }
    {   // conversion to q_0 .. q_{l-2}, forward transform, (acc - conv) D^-1
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l - 1;
        for (int i = 0; i < l - 1; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.y = y2.as<double>(); a.y_bs = (u64)(K + 1) * n; a.y_pos0 = 0; a.conv_a = K + 1; a.total = total; a.hat = tab->d_hat_f;
        a.acc = acc; a.acc_bs = (u64)ext_limbs * n; a.acc_pos_shift = 0; a.pinv_tab = dinv;
        a.out = out; a.out_bs = (u64)(l - 1) * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV_FINAL, log_n, a, tk, B * 2, st));
    }
    return HISA_OK;
}

// C and D for accumulators that carry the elementwise ends of the ModDown already (launch_inner_product_fold_fp):
// the special limbs hold sum * (P/p_m)^-1 as doubles, the limbs of q hold sum * P^-1 + addend.  out = ModDown + addend.
static int moddown_folded_fp(hisa_ctx* ctx, const u64* acc, size_t B, int l, u64* out, double* y2_ws) {
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, total = (int)ctx->total, ext_limbs = l + K, log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;
    const bool no_alloc = y2_ws != nullptr;
    Temp y2_t(ctx, B * 2 * (size_t)K * n * sizeof(double), !no_alloc);
    if (!no_alloc && !y2_t.ok()) return HISA_ERR_OOM;
    double* y2 = no_alloc ? y2_ws : y2_t.as<double>();
    FpArgs base = fp_base(ctx);
    if (no_alloc) { base.scratch = nullptr; base.scratch_polys = 0; base.no_pair = 1; }
    {   // C: batch entries are (ciphertext, b|a) pairs
        FpArgs a = base;
        FpTask tk = {};
        tk.period = K;
        for (int m = 0; m < K; m++) { tk.pos[m] = (int16_t)m; tk.prime[m] = (int16_t)(L + m); }
        a.in = acc; a.in_bs = (u64)ext_limbs * n; a.in_pos_shift = l;
        a.yout = y2; a.yout_bs = (u64)K * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_D_TO_Y, log_n, a, tk, B * 2, st));
    }
    {   // D
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l;
        for (int i = 0; i < l; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.y = y2; a.y_bs = (u64)K * n; a.y_pos0 = 0; a.conv_a = K; a.total = total; a.hat = ctx->d_moddown_hat_pin;
        a.acc = acc; a.acc_bs = (u64)ext_limbs * n; a.acc_pos_shift = 0;
        a.out = out; a.out_bs = (u64)l * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV_SUB, log_n, a, tk, B * 2, st));
    }
    return HISA_OK;
}

static int key_switch_finish_fp(hisa_ctx* ctx, const FpExt& x, const u64* d, u64 d_bs, u64 galois, int gather_ext, size_t B,
                                const SwitchKey& key, const u64* add, u64 add_bs, int add_polys, u64* out,
                                u64* acc_ws = nullptr, double* y2_ws = nullptr) {
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, l = x.l;
    const int ext_limbs = x.ext_limbs, log_n = (int)ctx->log_n;
    // acc_ws, y2_ws: the caller's memory for the accumulators and the ModDown input; both or neither
    if ((acc_ws == nullptr) != (y2_ws == nullptr)) return fail(ctx, HISA_ERR_ARG, "half a workspace");
    Temp acc_t(ctx, B * 2 * (size_t)ext_limbs * n * sizeof(u64), acc_ws == nullptr);
    if (!acc_ws && !acc_t.ok()) return HISA_ERR_OOM;
    u64* acc = acc_ws ? acc_ws : acc_t.u();
    double *post_q, *post_p;
    TRY(fp_post_tables(ctx, l, &post_q, &post_p, acc_ws != nullptr));
    // the addend is gathered through the same automorphism as the own-digit limbs
    IpFold fold = {ctx->d_pinv_f, post_p, add_polys > 0 ? add : nullptr, add_bs, (u64)l * n, add_polys};
    HIP_TRY(ctx, launch_inner_product_fold_fp(ctx->tabs.fprimes, x.extp, x.ext_bs, x.digits, l, K, L, alpha, key.data, total, d,
                                              d_bs, galois, gather_ext, acc, (u64)2 * ext_limbs * n, B, log_n, fold, ctx->stream));
    return moddown_folded_fp(ctx, acc, B, l, out, y2_ws);
}

// IP, C, D for n_steps rotations of the same B ciphertexts in one set of launches (entries rotation-major): a
// convolution's taps rotate few ciphertexts many times, and a launch over B entries alone would leave most of the chip
// idle.  out: [n_steps][B] ciphertexts.  Same arithmetic per entry as key_switch_finish_fp with gather_ext = 1.
static int key_switch_finish_steps_fp(hisa_ctx* ctx, const FpExt& x, const u64* d, u64 d_bs, const u64* galois,
                                      const SwitchKey* const* keys, int n_steps, size_t B, const u64* add, u64 add_bs, u64* out) {
    const size_t n = ctx->N, E = (size_t)n_steps * B;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, l = x.l;
    const int ext_limbs = x.ext_limbs, log_n = (int)ctx->log_n;
    hipStream_t st = ctx->stream;
    if (n_steps < 1 || n_steps > FP_MAX_STEPS) return fail(ctx, HISA_ERR_ARG, "bad rotation count");
    Temp acc(ctx, E * 2 * (size_t)ext_limbs * n * sizeof(u64));
    Temp y2(ctx, E * 2 * (size_t)K * n * sizeof(double));
    if (!acc.ok() || !y2.ok()) return HISA_ERR_OOM;
    double *post_q, *post_p;
    TRY(fp_post_tables(ctx, l, &post_q, &post_p, false));
    const FpArgs base = fp_base(ctx);
    IpSteps steps = {};
    for (int s = 0; s < n_steps; s++) { steps.key[s] = keys[s]->data; steps.galois[s] = (uint32_t)galois[s]; }
    HIP_TRY(ctx, launch_inner_product_steps_fp(ctx->tabs.fprimes, x.extp, x.ext_bs, x.digits, l, K, L, alpha, steps, n_steps,
                                               total, d, d_bs, acc.u(), (u64)2 * ext_limbs * n, B, log_n, st));
    {   // C
        FpArgs a = base;
        FpTask tk = {};
        tk.period = K;
        for (int m = 0; m < K; m++) { tk.pos[m] = (int16_t)m; tk.prime[m] = (int16_t)(L + m); }
        a.in = acc.u(); a.in_bs = (u64)ext_limbs * n; a.in_pos_shift = l; a.post = post_p;
        a.yout = y2.as<double>(); a.yout_bs = (u64)K * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_TO_Y, log_n, a, tk, E * 2, st));
    }
    {   // D
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l;
        for (int i = 0; i < l; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.y = y2.as<double>(); a.y_bs = (u64)K * n; a.y_pos0 = 0; a.conv_a = K; a.total = total; a.hat = ctx->moddown_tab->d_hat_f;
        a.acc = acc.u(); a.acc_bs = (u64)ext_limbs * n; a.acc_pos_shift = 0; a.pinv_tab = ctx->d_pinv_f;
        a.add = add; a.add_bs = add_bs; a.add_ps = (u64)l * n; a.add_div = 2; a.add_polys = 1;
        a.step_B = (int)B;
        for (int s = 0; s < n_steps; s++) a.galois_tab[s] = (uint32_t)galois[s];
        a.out = out; a.out_bs = (u64)l * n;
        HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV_FINAL, log_n, a, tk, E * 2, st));
    }
    return HISA_OK;
}

bool fused_key_switch_available(const hisa_ctx* ctx) { return ctx->tabs.fp_ok && ctx->dnum <= 8; }

// The key-switch accumulators -- before the division by P -- of n_steps rotations of B ciphertexts (cts: [B][2][l][N],
// ct_bs words apart): one decomposition + ModUp of c1, then per rotation the inner product with its key, gathered
// through its automorphism.  acc: [n_steps][B][2][l + K][N].  Every amount must be a real rotation with its key present.
// fold_c0: the first accumulator also takes P * sigma(c0) on the limbs of q, so that the rotated ciphertext is the
// ModDown of the accumulators alone (exactly: P sigma(c0) leaves the special limbs, and with them the conversion, as
// they are, and (x + P c) P^-1 = x P^-1 + c).
int rotation_accumulators_fp(hisa_ctx* ctx, const u64* cts, u64 ct_bs, size_t B, int l, const int32_t* steps, int n_steps,
                             u64* acc, bool fold_c0) {
    if (!fused_key_switch_available(ctx)) return fail(ctx, HISA_ERR_ARG, "no fused key-switch path for these parameters");
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, ext_limbs = l + K;
    std::vector<u64> gs(n_steps);
    for (int s = 0; s < n_steps; s++) {
        gs[s] = galois_of(ctx, steps[s]);
        if (gs[s] == 0) return fail(ctx, HISA_ERR_ARG, "rotation by a multiple of the slot count");
        if (ctx->keys.find(gs[s]) == ctx->keys.end())
            return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps[s], (unsigned long long)gs[s]);
    }
    FpExt x(ctx, B, l, K, alpha);
    if (!x.ok()) return HISA_ERR_OOM;
    const u64* c1 = cts + (size_t)l * n;
    TRY(key_switch_modup_fp(ctx, c1, ct_bs, 0, B, x));
    const u64 acc_bs = (u64)2 * ext_limbs * n;
    for (int g0 = 0; g0 < n_steps; g0 += FP_MAX_STEPS) {
        const int cnt = std::min(FP_MAX_STEPS, n_steps - g0);
        IpSteps st = {};
        for (int k = 0; k < cnt; k++) { st.key[k] = ctx->keys.find(gs[g0 + k])->second.data; st.galois[k] = (uint32_t)gs[g0 + k]; }
        HIP_TRY(ctx, launch_inner_product_steps_fp(ctx->tabs.fprimes, x.extp, x.ext_bs, x.digits, l, K, L, alpha, st, cnt, total,
                                                   c1, ct_bs, acc + (u64)g0 * B * acc_bs, acc_bs, B, (int)ctx->log_n, ctx->stream,
                                                   fold_c0 ? cts : nullptr, ctx->d_pmod));
    }
    return HISA_OK;
}

int rotate_sum_fp(hisa_ctx* ctx, const u64* rot, u64 ct_bs, int n_steps, const int32_t* steps, size_t Bn, int l,
                  const u64* plain, u64 plain_bs, u64* out, bool shared_input, bool rescale) {
    if (!fused_key_switch_available(ctx)) return fail(ctx, HISA_ERR_ARG, "no fused key-switch path for these parameters");
    if (n_steps < 1 || n_steps > FP_MAX_STEPS || Bn == 0 || l < 1) return fail(ctx, HISA_ERR_ARG, "bad rotation sum");
    const size_t n = ctx->N;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, ext_limbs = l + K;
    if (ct_bs < (u64)2 * l * n || (plain && plain_bs < (u64)2 * l * n)) return fail(ctx, HISA_ERR_ARG, "bad rotation sum strides");
    IpSteps st = {};
    GaloisTab tab = {};
    for (int s = 0; s < n_steps; s++) {
        const u64 g = galois_of(ctx, steps[s]);
        if (g == 0) return fail(ctx, HISA_ERR_ARG, "rotation by a multiple of the slot count");
        if (t_analysis) {
            const int32_t half = (int32_t)(ctx->N / 2);
            t_analysis->steps.insert(((steps[s] % half) + half) % half);
            continue;
        }
        auto it = ctx->keys.find(g);
        if (it == ctx->keys.end())
            return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps[s], (unsigned long long)g);
        st.key[s] = it->second.data;
        st.galois[s] = (uint32_t)g;
        tab.g[s] = (uint32_t)g;
    }
    if (t_analysis) {
        TALLY(rot_left, HISA_OP_ROT_LEFT, (u64)n_steps * Bn, l);
        TALLY(rot_summed, HISA_OP_ROT_SUMMED, (u64)n_steps * Bn, l);
        if (shared_input) TALLY(rot_shared, HISA_OP_ROT_SHARED, (u64)(n_steps - 1) * Bn, l);
        TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, 1, l);
        if (rescale) TALLY(rescale, HISA_OP_RESCALE, Bn, l);
        return HISA_OK;
    }
    if (rescale && l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "no level to rescale into");
    const size_t E = shared_input ? Bn : (size_t)n_steps * Bn;
    FpExt x(ctx, E, l, K, alpha);
    Temp acc(ctx, Bn * 2 * (size_t)ext_limbs * n * sizeof(u64));
    Temp addend(ctx, Bn * 2 * (size_t)l * n * sizeof(u64));
    if (!x.ok() || !acc.ok() || !addend.ok()) return HISA_ERR_OOM;
    const u64* c1 = rot + (size_t)l * n;
    TRY(key_switch_modup_fp(ctx, c1, ct_bs, 0, E, x));
    HIP_TRY(ctx, launch_inner_product_sum_fp(ctx->tabs.fprimes, x.extp, x.ext_bs, x.digits, l, K, L, alpha, st, n_steps, total,
                                             c1, ct_bs, acc.u(), (u64)2 * ext_limbs * n, Bn, shared_input ? 1 : 0, (int)ctx->log_n,
                                             ctx->stream));
    HIP_TRY(ctx, launch_automorph_sum(ctx->d_primes, rot, ct_bs, n_steps, tab, plain, plain_bs, addend.u(), (u64)2 * l * n, Bn,
                                      shared_input ? 1 : 0, l,
                                      (int)ctx->log_n, ctx->stream));
    if (rescale) return moddown_rescale_fp(ctx, acc.u(), Bn, l, addend.u(), (u64)2 * l * n, 2, out);
    return moddown_add_fp(ctx, acc.u(), Bn, l, addend.u(), (u64)2 * l * n, 2, 0, out);
}

int relinearize_rescale_fp(hisa_ctx* ctx, const u64* cts3, u64 stride, size_t n_cts, int l, u64* out) {
    if (!fused_key_switch_available(ctx)) return fail(ctx, HISA_ERR_ARG, "no fused key-switch path for these parameters");
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "no level to rescale into");
    if (t_analysis) {
        TALLY(relinearize, HISA_OP_RELINEARIZE, n_cts, l);
        TALLY(rescale, HISA_OP_RESCALE, n_cts, l);
        TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, 1, l);
        return HISA_OK;
    }
    auto it = ctx->keys.find(0);
    if (it == ctx->keys.end()) return fail(ctx, HISA_ERR_NO_KEY, "no relinearisation key: call hisa_keygen");
    const size_t n = ctx->N, lw = (size_t)l * n;
    const int K = (int)ctx->K, L = (int)ctx->L, alpha = (int)ctx->alpha, total = (int)ctx->total, ext_limbs = l + K;
    if (stride < 3 * lw) return fail(ctx, HISA_ERR_ARG, "bad stride");
    FpExt x(ctx, n_cts, l, K, alpha);
    Temp acc(ctx, n_cts * 2 * (size_t)ext_limbs * n * sizeof(u64));
    if (!x.ok() || !acc.ok()) return HISA_ERR_OOM;
    const u64* d2 = cts3 + 2 * lw;
    TRY(key_switch_modup_fp(ctx, d2, stride, 0, n_cts, x));
    HIP_TRY(ctx, launch_inner_product_fp(ctx->tabs.fprimes, x.extp, x.ext_bs, x.digits, l, K, L, alpha, it->second.data, total, d2,
                                         stride, 0, 0, acc.u(), (u64)2 * ext_limbs * n, n_cts, (int)ctx->log_n, ctx->stream));
    return moddown_rescale_fp(ctx, acc.u(), n_cts, l, cts3, stride, 2, out);
}

extern "C" int hisa_set_fused_rescale(hisa_ctx* ctx, uint32_t on) {
    if (!ctx) return HISA_ERR_ARG;
    if (on > 1) return fail(ctx, HISA_ERR_ARG, "on is 0 or 1");
    if (on && !fused_key_switch_available(ctx))
        return fail(ctx, HISA_ERR_ARG, "the combined division needs the fused key-switch path (N >= 2^12, every prime below 2^50, dnum <= 8)");
    ctx->fused_rescale = on;
    return HISA_OK;
}

extern "C" int hisa_rot_left_sum_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n_out, const int32_t* steps,
                                       size_t n_terms, hisa_ct** out) {
    if (!ctx || !out || !steps || n_terms == 0 || n_out == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, in, n_out * n_terms, 2));
    if (!fused_key_switch_available(ctx))
        return fail(ctx, HISA_ERR_ARG, "sums of rotations need the fused key-switch path (N >= 2^12, every prime below 2^50, dnum <= 8)");
    for (size_t i = 1; i < n_out * n_terms; i++)
        if (fabs(in[i]->scale - in[0]->scale) > 1e-9 * fabs(in[0]->scale)) return fail(ctx, HISA_ERR_SCALE_MISMATCH, "terms of different scales");
    // rotated terms first, in order; the unrotated one (if any) apart
    std::vector<int32_t> rot_steps;
    std::vector<const hisa_ct*> rot_in, plain_in;
    for (size_t s = 0; s < n_terms; s++) {
        const u64 g = galois_of(ctx, steps[s]);
        if (g == 0) {
            if (!plain_in.empty()) return fail(ctx, HISA_ERR_ARG, "more than one term without a rotation");
            plain_in.assign(in + s * n_out, in + (s + 1) * n_out);
            continue;
        }
        if (!t_analysis && ctx->keys.find(g) == ctx->keys.end())
            return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps[s], (unsigned long long)g);
        rot_steps.push_back(steps[s]);
        rot_in.insert(rot_in.end(), in + s * n_out, in + (s + 1) * n_out);
    }
    if (rot_steps.size() > FP_MAX_STEPS) return fail(ctx, HISA_ERR_ARG, "at most %d rotated terms", FP_MAX_STEPS);
    // every rotated term of an output the same ciphertext: one decomposition per output serves all its rotations
    bool shared_input = rot_steps.size() > 1;
    for (size_t i = n_out; i < rot_in.size() && shared_input; i++) shared_input = rot_in[i] == rot_in[i % n_out];
    if (shared_input) rot_in.resize(n_out);
    const int l = (int)in[0]->limbs;
    TRY(alloc_ct_batch(ctx, n_out, 2, (uint32_t)l, in[0]->scale, out));
    int rc = HISA_OK;
    BatchIn br = {}, bp = {};
    if (t_analysis) {   // a dry run moves no data
        br.stride = bp.stride = ct_words(ctx, 2, l);
    } else {
        if (!plain_in.empty()) rc = gather_batch(ctx, plain_in.data(), n_out, &bp);
        if (rc == HISA_OK && !rot_in.empty()) rc = gather_batch(ctx, rot_in.data(), rot_in.size(), &br);
    }
    if (rc == HISA_OK) {
        if (rot_in.empty()) {   // nothing rotates: a copy of the one term
            hipError_t e = hipSuccess;
            for (size_t b = 0; b < n_out && e == hipSuccess && !t_analysis; b++)
                e = hipMemcpyAsync(out[b]->data, plain_in[b]->data, ct_words(ctx, 2, l) * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "copy: %s", hipGetErrorString(e));
        } else {
            rc = rotate_sum_fp(ctx, br.base, br.stride, (int)rot_steps.size(), rot_steps.data(), n_out, l,
                               plain_in.empty() ? nullptr : bp.base, bp.stride, out[0]->data, shared_input);
        }
    }
    dev_release(ctx, br.tmp);
    dev_release(ctx, bp.tmp);
    if (rc != HISA_OK)
        for (size_t b = 0; b < n_out; b++) { hisa_free(ctx, out[b]); out[b] = nullptr; }
    return rc;
}

static int key_switch_core_fp(hisa_ctx* ctx, const u64* d, u64 d_bs, u64 galois, size_t B, int l, const SwitchKey& key,
                              const u64* add, u64 add_bs, int add_polys, u64* out) {
    FpExt x(ctx, B, l, (int)ctx->K, (int)ctx->alpha);
    if (!x.ok()) return HISA_ERR_OOM;
    TRY(key_switch_modup_fp(ctx, d, d_bs, galois, B, x));
    return key_switch_finish_fp(ctx, x, d, d_bs, galois, 0, B, key, add, add_bs, add_polys, out);
}

extern "C" int hisa_analysis_begin(hisa_ctx* ctx) {
    if (!ctx) return HISA_ERR_ARG;
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "a context of this thread is already in analysis mode");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->analysis = new Analysis();
    t_analysis = ctx->analysis;
    return HISA_OK;
}

extern "C" int hisa_analysis_end(hisa_ctx* ctx, hisa_op_counts* counts, int32_t* rot_steps, size_t cap, size_t* n) {
    if (!ctx) return HISA_ERR_ARG;
    if (!ctx->analysis || t_analysis != ctx->analysis) return fail(ctx, HISA_ERR_ARG, "the context is not in analysis mode");
    Analysis* a = ctx->analysis;
    ctx->analysis = nullptr;
    t_analysis = nullptr;
    int rc = HISA_OK;
    if (counts) *counts = a->c;
    if (n) *n = a->steps.size();
    if (rot_steps) {
        size_t i = 0;
        for (int32_t s : a->steps) {
            if (i >= cap) { rc = fail(ctx, HISA_ERR_ARG, "%zu rotation amounts do not fit %zu entries", a->steps.size(), cap); break; }
            rot_steps[i++] = s;
        }
    }
    delete a;
    return rc;
}

extern "C" int hisa_rot_left_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n, int32_t steps, hisa_ct** out) {
    if (!ctx || !out) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, in, n, 2));
    const u64 g = galois_of(ctx, steps);
    const int l = (int)in[0]->limbs;
    if (g == 0) {  // rotation by a multiple of N/2: a copy, no key needed
        TRY(alloc_ct_batch(ctx, n, 2, (uint32_t)l, 0.0, out));
        for (size_t i = 0; i < n; i++) {
            out[i]->scale = in[i]->scale;
            HIP_TRY(ctx, hipMemcpyAsync(out[i]->data, in[i]->data, ct_words(ctx, 2, l) * sizeof(u64), hipMemcpyDeviceToDevice,
                                        ctx->stream));
        }
        return HISA_OK;
    }
    if (t_analysis) {   // dry run: note the amount, hand out ciphertexts of the right level and scale
        const int32_t half = (int32_t)(ctx->N / 2);
        t_analysis->steps.insert(((steps % half) + half) % half);
        TALLY(rot_left, HISA_OP_ROT_LEFT, n, l);
        TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, 1, l);
        TRY(alloc_ct_batch(ctx, n, 2, (uint32_t)l, 0.0, out));
        for (size_t i = 0; i < n; i++) out[i]->scale = in[i]->scale;
        return HISA_OK;
    }
    auto it = ctx->keys.find(g);
    if (it == ctx->keys.end()) return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps,
                                           (unsigned long long)g);
    BatchIn bi;
    TRY(gather_batch(ctx, in, n, &bi));
    const size_t nn = ctx->N, lw = (size_t)l * nn;
    int rc = HISA_OK;
    if (ctx->tabs.fp_ok && ctx->dnum <= 8) {
        // fused fp64 pipeline: both automorphisms are gathers inside its first and last kernels
        rc = alloc_ct_batch(ctx, n, 2, (uint32_t)l, 0.0, out);
        if (rc == HISA_OK) {
            for (size_t i = 0; i < n; i++) out[i]->scale = in[i]->scale;
            rc = key_switch_core_fp(ctx, bi.base + lw, bi.stride, g, n, l, it->second, bi.base, bi.stride, 1, out[0]->data);
        }
    } else {
        // sigma_g(c1) in NTT form (a gather); sigma_g(c0) is gathered inside the last kernel
        Temp r1(ctx, n * lw * sizeof(u64));
        if (!r1.ok()) rc = HISA_ERR_OOM;
        if (rc == HISA_OK) {
            hipError_t e = launch_automorph_ntt(bi.base + lw, bi.stride, r1.u(), lw, g, l, n, (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "automorph: %s", hipGetErrorString(e));
        }
        if (rc == HISA_OK) rc = alloc_ct_batch(ctx, n, 2, (uint32_t)l, 0.0, out);
        if (rc == HISA_OK) {
            for (size_t i = 0; i < n; i++) out[i]->scale = in[i]->scale;
            rc = key_switch_core(ctx, r1.u(), lw, n, l, it->second, bi.base, bi.stride, 1, g, out[0]->data);
        }
    }
    dev_release(ctx, bi.tmp);
    return rc;
}

extern "C" int hisa_rot_left_hoisted_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n, const int32_t* steps,
                                           size_t n_steps, hisa_ct** out) {
    if (!ctx || !out || !steps || n_steps == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_batch_shape(ctx, in, n, 2));
    for (size_t s = 0; s < n * n_steps; s++) out[s] = nullptr;
    // every key must be there before any work is queued
    std::vector<u64> gs(n_steps);
    size_t switched = 0;
    for (size_t s = 0; s < n_steps; s++) {
        gs[s] = galois_of(ctx, steps[s]);
        if (gs[s] == 0) continue;
        switched++;
        if (!t_analysis && ctx->keys.find(gs[s]) == ctx->keys.end())
            return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps[s],
                        (unsigned long long)gs[s]);
    }
    const int l = (int)in[0]->limbs;
    int rc = HISA_OK;
    if (t_analysis) {
        for (size_t s = 0; s < n_steps && rc == HISA_OK; s++) rc = hisa_rot_left_batch(ctx, in, n, steps[s], out + s * n);
        if (rc == HISA_OK && switched >= 2 && ctx->tabs.fp_ok && ctx->dnum <= 8) {
            // one decomposition, then one set of launches per group of rotations (as in the branch below)
            const size_t group = std::max<size_t>(1, std::min<size_t>(FP_MAX_STEPS, 1024 / n));
            TALLY(rot_shared, HISA_OP_ROT_SHARED, (switched - 1) * n, l);
            t_analysis->c.key_switch_calls -= switched;
            t_analysis->c.limb_sum[HISA_OP_KEY_SWITCH_CALLS] -= (u64)switched * l;
            t_analysis->c.limb_sq_sum[HISA_OP_KEY_SWITCH_CALLS] -= (u64)switched * l * l;
            TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, (switched + group - 1) / group, l);
        }
    } else if (switched < 2 || !(ctx->tabs.fp_ok && ctx->dnum <= 8)) {   // nothing to share, or no fused path: one by one
        for (size_t s = 0; s < n_steps && rc == HISA_OK; s++) rc = hisa_rot_left_batch(ctx, in, n, steps[s], out + s * n);
    } else {
        BatchIn bi;
        TRY(gather_batch(ctx, in, n, &bi));
        const size_t lw = (size_t)l * ctx->N;
        {
            FpExt x(ctx, n, l, (int)ctx->K, (int)ctx->alpha);
            if (!x.ok()) rc = HISA_ERR_OOM;
            if (rc == HISA_OK) rc = key_switch_modup_fp(ctx, bi.base + lw, bi.stride, 0, n, x);
            // rotations by a multiple of the slot count are copies; the others go through the key switch in groups
            // of at most FP_MAX_STEPS rotations (and a bounded number of entries) per set of launches
            std::vector<size_t> sw;
            for (size_t s = 0; s < n_steps && rc == HISA_OK; s++) {
                if (gs[s] == 0) rc = hisa_rot_left_batch(ctx, in, n, steps[s], out + s * n);
                else sw.push_back(s);
            }
            const size_t group = std::max<size_t>(1, std::min<size_t>(FP_MAX_STEPS, 1024 / n));
            for (size_t g0 = 0; g0 < sw.size() && rc == HISA_OK; g0 += group) {
                const size_t cnt = std::min(group, sw.size() - g0);
                std::vector<hisa_ct*> fresh(cnt * n, nullptr);
                rc = alloc_ct_batch(ctx, cnt * n, 2, (uint32_t)l, 0.0, fresh.data());
                if (rc != HISA_OK) break;
                u64 gal[FP_MAX_STEPS];
                const SwitchKey* keys[FP_MAX_STEPS];
                for (size_t k = 0; k < cnt; k++) {
                    gal[k] = gs[sw[g0 + k]];
                    keys[k] = &ctx->keys.find(gal[k])->second;
                    for (size_t i = 0; i < n; i++) {
                        fresh[k * n + i]->scale = in[i]->scale;
                        out[sw[g0 + k] * n + i] = fresh[k * n + i];
                    }
                }
                rc = key_switch_finish_steps_fp(ctx, x, bi.base + lw, bi.stride, gal, keys, (int)cnt, n, bi.base, bi.stride,
                                                fresh[0]->data);
            }
        }
        dev_release(ctx, bi.tmp);
    }
    if (rc != HISA_OK)
        for (size_t s = 0; s < n * n_steps; s++)
            if (out[s]) { hisa_free(ctx, out[s]); out[s] = nullptr; }
    return rc;
}

extern "C" int hisa_rot_left(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct** out) {
    return hisa_rot_left_batch(ctx, &a, 1, steps, out);
}

extern "C" int hisa_rot_right(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct** out) {
    if (!ctx) return HISA_ERR_ARG;
    const i64 slots = ctx->N / 2;
    i64 r = (i64)steps % slots;
    if (r < 0) r += slots;
    return hisa_rot_left_batch(ctx, &a, 1, (int32_t)((slots - r) % slots), out);
}

extern "C" int hisa_rot_left_assign(hisa_ctx* ctx, hisa_ct* a, int32_t steps) {
    hisa_ct* tmp = nullptr;
    const hisa_ct* ca = a;
    TRY(hisa_rot_left_batch(ctx, &ca, 1, steps, &tmp));
    adopt(ctx, a, tmp);
    return HISA_OK;
}

extern "C" int hisa_rot_right_assign(hisa_ctx* ctx, hisa_ct* a, int32_t steps) {
    hisa_ct* tmp = nullptr;
    TRY(hisa_rot_right(ctx, a, steps, &tmp));
    adopt(ctx, a, tmp);
    return HISA_OK;
}

// rotLeft of one ciphertext into an existing one, for callers that cannot allocate: the intermediates live in the
// library's static scratch array, the small tables were built with the context, and the conversion kernels run one
// target limb per task (the paired form parks partial sums in a buffer of its own).  Same launches otherwise, so the
// result is bit for bit hisa_rot_left's.
extern "C" int hisa_rot_left_noalloc(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct* out) {
    if (!ctx) return HISA_ERR_ARG;
    if (!valid_ct(a) || !valid_ct(out)) return fail(ctx, HISA_ERR_ARG, "not a ciphertext");
    if (a->polys != 2 || out->polys != 2) return fail(ctx, HISA_ERR_SIZE, "rotation needs two-polynomial ciphertexts");
    if (a->limbs != out->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "output has %u limbs, input %u", out->limbs, a->limbs);
    const size_t n = ctx->N;
    const int l = (int)a->limbs, K = (int)ctx->K, alpha = (int)ctx->alpha;
    const size_t words = ct_words(ctx, 2, (uint32_t)l);
    if (a->data < out->data + words && out->data < a->data + words)
        return fail(ctx, HISA_ERR_ARG, "input and output overlap");
    const u64 g = galois_of(ctx, steps);
    if (t_analysis) {
        if (g) {
            const int32_t half = (int32_t)(ctx->N / 2);
            t_analysis->steps.insert(((steps % half) + half) % half);
            TALLY(rot_left, HISA_OP_ROT_LEFT, 1, l);
            TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, 1, l);
        }
        out->scale = a->scale;
        return HISA_OK;
    }
    if (g == 0) {
        HIP_TRY(ctx, hipMemcpyAsync(out->data, a->data, words * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream));
        out->scale = a->scale;
        return HISA_OK;
    }
    if (!fused_key_switch_available(ctx))
        return fail(ctx, HISA_ERR_ARG, "hisa_rot_left_noalloc needs 2^12 <= N <= 2^15, every prime below 2^50 and dnum <= 8");
    if (g_prof_on) return fail(ctx, HISA_ERR_ARG, "per-kernel timing creates events; switch it off for hisa_rot_left_noalloc");
    auto it = ctx->keys.find(g);
    if (it == ctx->keys.end()) return fail(ctx, HISA_ERR_NO_KEY, "no rotation key for %d slots (galois element %llu)", steps,
                                           (unsigned long long)g);
    int dev = -1;
    HIP_TRY(ctx, hipGetDevice(&dev));
    if (dev != ctx->device || !ctx->noalloc_ws) return fail(ctx, HISA_ERR_ARG, "the context lives on device %d, current is %d", ctx->device, dev);
    // layout of the scratch array: y | ext | acc | y2, each 256-byte aligned
    auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
    const size_t y_b = up(FpExt::y_bytes(ctx, 1, l)), ext_b = up(FpExt::ext_bytes(ctx, 1, l, K, alpha));
    const size_t acc_b = up((size_t)2 * (l + K) * n * sizeof(u64)), y2_b = up((size_t)2 * K * n * sizeof(double));
    const size_t need = y_b + ext_b + acc_b + y2_b;
    if (need > (size_t)HISA_NOALLOC_SCRATCH_BYTES)
        return fail(ctx, HISA_ERR_SIZE, "a rotation at N = %zu, %d limbs, %d special primes needs %zu bytes of scratch; the static array holds %zu",
                    n, l, K, need, (size_t)HISA_NOALLOC_SCRATCH_BYTES);
    unsigned char* ws = (unsigned char*)ctx->noalloc_ws;
    FpExt x(ctx, l, K, alpha, (double*)ws, (double*)(ws + y_b));
    const size_t lw = (size_t)l * n;
    TRY(key_switch_modup_fp(ctx, a->data + lw, words, g, 1, x, true));
    TRY(key_switch_finish_fp(ctx, x, a->data + lw, words, g, 0, 1, it->second, a->data, words, 1, out->data,
                             (u64*)(ws + y_b + ext_b), (double*)(ws + y_b + ext_b + acc_b)));
    out->scale = a->scale;
    return HISA_OK;
}

extern "C" int hisa_relinearize_batch(hisa_ctx* ctx, hisa_ct* const* cts, size_t n) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_batch_shape(ctx, (const hisa_ct* const*)cts, n, 0));
    if (cts[0]->polys == 2) return HISA_OK;
    if (cts[0]->polys != 3) return fail(ctx, HISA_ERR_SIZE, "relinearize needs 2 or 3 polynomials");
    if (t_analysis) {
        TALLY(relinearize, HISA_OP_RELINEARIZE, n, cts[0]->limbs);
        TALLY(key_switch_calls, HISA_OP_KEY_SWITCH_CALLS, 1, cts[0]->limbs);
        std::vector<hisa_ct*> two(n);
        TRY(alloc_ct_batch(ctx, n, 2, cts[0]->limbs, 0.0, two.data()));
        for (size_t i = 0; i < n; i++) {
            two[i]->scale = cts[i]->scale;
            adopt(ctx, cts[i], two[i]);
        }
        return HISA_OK;
    }
    auto it = ctx->keys.find(0);
    if (it == ctx->keys.end()) return fail(ctx, HISA_ERR_NO_KEY, "no relinearisation key: call hisa_keygen");
    const int l = (int)cts[0]->limbs;
    const size_t lw = (size_t)l * ctx->N;
    BatchIn bi;
    TRY(gather_batch(ctx, (const hisa_ct* const*)cts, n, &bi));
    std::vector<hisa_ct*> fresh(n);
    int rc = alloc_ct_batch(ctx, n, 2, (uint32_t)l, 0.0, fresh.data());
    if (rc == HISA_OK) {
        if (ctx->tabs.fp_ok && ctx->dnum <= 8)
            rc = key_switch_core_fp(ctx, bi.base + 2 * lw, bi.stride, 0, n, l, it->second, bi.base, bi.stride, 2, fresh[0]->data);
        else
            rc = key_switch_core(ctx, bi.base + 2 * lw, bi.stride, n, l, it->second, bi.base, bi.stride, 2, 0, fresh[0]->data);
        for (size_t i = 0; i < n; i++) {
            fresh[i]->scale = cts[i]->scale;
            if (rc == HISA_OK) adopt(ctx, cts[i], fresh[i]);
            else hisa_free(ctx, fresh[i]);
        }
    }
    dev_release(ctx, bi.tmp);
    return rc;
}

extern "C" int hisa_relinearize(hisa_ctx* ctx, hisa_ct* ct) { return hisa_relinearize_batch(ctx, &ct, 1); }

extern "C" int hisa_mul(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out) {
    if (!out) return fail(ctx, HISA_ERR_ARG, "null out");
    TRY(hisa_mul_no_relin(ctx, a, b, out));
    int rc = hisa_relinearize(ctx, *out);
    if (rc != HISA_OK) { hisa_free(ctx, *out); *out = nullptr; }
    return rc;
}

extern "C" int hisa_mul_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b) {
    hisa_ct* tmp = nullptr;
    TRY(hisa_mul(ctx, a, b, &tmp));
    adopt(ctx, a, tmp);
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// division profile
// ---------------------------------------------------------------------------
extern "C" int hisa_max_scalar_div(hisa_ctx* ctx, const hisa_ct* ct, double ub, uint64_t* d) {
    if (!ctx || !valid_ct(ct) || !d) return fail(ctx, HISA_ERR_ARG, "bad argument");
    *d = 1;
    if (ct->limbs > 1 && (double)ctx->mod[ct->limbs - 1] < ub) *d = ctx->mod[ct->limbs - 1];
    return HISA_OK;
}

// Constants of the fp64 rescale at level l, device resident: `total` ones (the base conversion from a one-prime
// basis has hat = 1), then q_{l-1}^-1 mod q_i as centred doubles for i < l-1.
static int fp_rescale_tables(hisa_ctx* ctx, int l, double** ones, double** qlinv) {
    const u64 KEY = 8192 + (u64)l;
    auto it = ctx->aux.find(KEY);
    if (it == ctx->aux.end()) {
        std::vector<double> t((size_t)ctx->total + l, 1.0);
        for (int i = 0; i < l - 1; i++)
            t[ctx->total + i] = centred_double(hm::inv(ctx->mod[l - 1] % ctx->mod[i], ctx->mod[i]), ctx->mod[i]);
        double* d = nullptr;
        HIP_TRY(ctx, upload(&d, t));
        it = ctx->aux.emplace(KEY, SwitchKey{new DevBlock{d, t.size() * sizeof(double), 1}, (u64*)d}).first;
    }
    *ones = (double*)it->second.data;
    *qlinv = (double*)it->second.data + ctx->total;
    return HISA_OK;
}

// Rescale with the fused fp64 kernels: the last limb goes to centred coefficient form (one inverse transform per
// polynomial), and one launch reduces it to every remaining prime, transforms it and forms (c_i - r) q_{l-1}^-1.
// It is the special-prime division of the key switch with a single "special" prime q_{l-1}.
static int rescale_core_fp(hisa_ctx* ctx, const u64* in, size_t n_bp, int l, u64* out) {
    const size_t nn = ctx->N;
    const int log_n = (int)ctx->log_n;
    Temp y(ctx, n_bp * nn * sizeof(double));
    if (!y.ok()) return HISA_ERR_OOM;
    double *ones, *qlinv;
    TRY(fp_rescale_tables(ctx, l, &ones, &qlinv));
    const FpArgs base = fp_base(ctx);
    {
        FpArgs a = base;
        FpTask tk = {};
        tk.period = 1; tk.pos[0] = 0; tk.prime[0] = (int16_t)(l - 1);
        a.in = in; a.in_bs = (u64)l * nn; a.in_pos_shift = l - 1; a.post = ones;
        a.yout = y.as<double>(); a.yout_bs = nn;
        HIP_TRY(ctx, launch_ntt_fp(FP_INV_TO_Y, log_n, a, tk, n_bp, ctx->stream));
    }
    {
        FpArgs a = base;
        FpTask tk = {};
        tk.period = l - 1;
        for (int i = 0; i < l - 1; i++) { tk.pos[i] = (int16_t)i; tk.prime[i] = (int16_t)i; }
        a.y = y.as<double>(); a.y_bs = nn; a.y_pos0 = 0; a.conv_a = 1; a.total = (int)ctx->total; a.hat = ones;
        a.acc = in; a.acc_bs = (u64)l * nn; a.acc_pos_shift = 0; a.pinv_tab = qlinv;
        a.out = out; a.out_bs = (u64)(l - 1) * nn;
        HIP_TRY(ctx, launch_ntt_fp(FP_FWD_CONV_FINAL, log_n, a, tk, n_bp, ctx->stream));
    }
    return HISA_OK;
}

extern "C" int hisa_rescale_batch(hisa_ctx* ctx, hisa_ct* const* cts, size_t n) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_batch_shape(ctx, (const hisa_ct* const*)cts, n, 0));
    const int l = (int)cts[0]->limbs, polys = (int)cts[0]->polys;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "rescale of a one-limb ciphertext");
    if (t_analysis) TALLY(rescale, HISA_OP_RESCALE, n, l);
    const size_t nn = ctx->N, n_bp = n * polys;
    BatchIn bi;
    TRY(gather_batch(ctx, (const hisa_ct* const*)cts, n, &bi));
    int rc = HISA_OK;
    std::vector<hisa_ct*> fresh(n);
    if (ctx->tabs.fp_ok) {
        rc = alloc_ct_batch(ctx, n, (uint32_t)polys, (uint32_t)(l - 1), 0.0, fresh.data());
        if (rc == HISA_OK) {
            rc = rescale_core_fp(ctx, bi.base, n_bp, l, fresh[0]->data);
            for (size_t i = 0; i < n; i++) {
                fresh[i]->scale = cts[i]->scale / (double)ctx->mod[l - 1];
                if (rc == HISA_OK) adopt(ctx, cts[i], fresh[i]);
                else hisa_free(ctx, fresh[i]);
            }
        }
    } else {
        Temp last(ctx, n_bp * nn * sizeof(u64));
        Temp r(ctx, n_bp * (size_t)(l - 1) * nn * sizeof(u64));
        if (!last.ok() || !r.ok()) rc = HISA_ERR_OOM;
        if (rc == HISA_OK) rc = alloc_ct_batch(ctx, n, (uint32_t)polys, (uint32_t)(l - 1), 0.0, fresh.data());
        if (rc == HISA_OK) {
            hipError_t e;
            PolyMap pm = {};
            pm.period = l;
            for (int i = 0; i < l; i++) pm.prime_of[i] = i == l - 1 ? (int16_t)(l - 1) : (int16_t)-1;
            InttExtra ex = {};
            ex.in = bi.base; ex.in_batch_stride = (u64)l * nn; ex.out_entry0 = l - 1;
            e = launch_intt(ctx->tabs, (int)ctx->log_n, last.u(), nn, (int)(n_bp * l), pm, &ex, ctx->stream);
            if (e == hipSuccess) e = launch_rescale_spread(ctx->d_primes, last.u(), r.u(), l, n_bp, (int)ctx->log_n, ctx->stream);
            if (e == hipSuccess)
                e = launch_ntt(ctx->tabs, (int)ctx->log_n, r.u(), (u64)(l - 1) * nn, (int)(n_bp * (l - 1)), identity_map(l - 1),
                               ctx->stream);
            u64 qlinv[HISA_MAX_Q], qlinv_sh[HISA_MAX_Q];
            for (int i = 0; i < l - 1; i++) {
                qlinv[i] = hm::inv(ctx->mod[l - 1] % ctx->mod[i], ctx->mod[i]);
                qlinv_sh[i] = hm::shoup(qlinv[i], ctx->mod[i]);
            }
            if (e == hipSuccess)
                e = launch_rescale_final(ctx->d_primes, bi.base, r.u(), qlinv, qlinv_sh, fresh[0]->data, l, n_bp, (int)ctx->log_n,
                                         ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "rescale: %s", hipGetErrorString(e));
            for (size_t i = 0; i < n; i++) {
                fresh[i]->scale = cts[i]->scale / (double)ctx->mod[l - 1];
                if (rc == HISA_OK) adopt(ctx, cts[i], fresh[i]);
                else hisa_free(ctx, fresh[i]);
            }
        }
    }
    dev_release(ctx, bi.tmp);
    return rc;
}

extern "C" int hisa_rescale(hisa_ctx* ctx, hisa_ct* ct) { return hisa_rescale_batch(ctx, &ct, 1); }

extern "C" int hisa_div_scalar(hisa_ctx* ctx, hisa_ct* ct, uint64_t d) {
    if (!ctx || !valid_ct(ct)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (d == 1) return HISA_OK;
    if (ct->limbs < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "no modulus left to divide by");
    if (d != ctx->mod[ct->limbs - 1])
        return fail(ctx, HISA_ERR_BAD_DIVISOR, "divisor %llu is not the last modulus %llu", (unsigned long long)d,
                    (unsigned long long)ctx->mod[ct->limbs - 1]);
    return hisa_rescale(ctx, ct);
}

// ---------------------------------------------------------------------------
// parity / debug surface
// ---------------------------------------------------------------------------
extern "C" int hisa_get_primes(hisa_ctx* ctx, uint64_t* q, uint64_t* p) {
    if (!ctx) return HISA_ERR_ARG;
    if (q) for (uint32_t i = 0; i < ctx->L; i++) q[i] = ctx->mod[i];
    if (p) for (uint32_t i = 0; i < ctx->K; i++) p[i] = ctx->mod[ctx->L + i];
    return HISA_OK;
}

extern "C" int hisa_get_alpha(hisa_ctx* ctx, uint32_t* alpha) {
    if (!ctx || !alpha) return HISA_ERR_ARG;
    *alpha = ctx->alpha;
    return HISA_OK;
}

extern "C" int hisa_ct_info(const hisa_ct* ct, uint32_t* limbs, uint32_t* polys, double* scale) {
    if (!valid_ct(ct)) return HISA_ERR_ARG;
    if (limbs) *limbs = ct->limbs;
    if (polys) *polys = ct->polys;
    if (scale) *scale = ct->scale;
    return HISA_OK;
}

extern "C" int hisa_ct_device_ptr(const hisa_ct* ct, uint64_t** dev) {
    if (!valid_ct(ct) || !dev) return HISA_ERR_ARG;
    *dev = ct->data;
    return HISA_OK;
}

extern "C" int hisa_ct_export(hisa_ctx* ctx, const hisa_ct* ct, uint64_t* host) {
    if (!ctx || !valid_ct(ct) || !host) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const size_t words = ct_words(ctx, ct->polys, ct->limbs);
    Temp co(ctx, words * sizeof(u64));
    if (!co.ok()) return HISA_ERR_OOM;
    InttExtra ex = {};
    ex.in = ct->data; ex.in_batch_stride = (u64)ct->limbs * ctx->N;
    HIP_TRY(ctx, launch_intt(ctx->tabs, (int)ctx->log_n, co.u(), (u64)ct->limbs * ctx->N, (int)(ct->polys * ct->limbs),
                             identity_map((int)ct->limbs), &ex, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(host, co.u(), words * sizeof(u64), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_ct_import_batch(hisa_ctx* ctx, const uint64_t* host, size_t n, uint32_t polys, uint32_t limbs,
                                    double scale, hisa_ct** out) {
    if (!ctx || !host || !out || n == 0 || polys < 1 || polys > 3 || limbs < 1 || limbs > ctx->L)
        return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_ct_batch(ctx, n, polys, limbs, scale, out));
    const size_t words = n * ct_words(ctx, polys, limbs);
    HIP_TRY(ctx, hipMemcpyAsync(out[0]->data, host, words * sizeof(u64), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, out[0]->data, (u64)limbs * ctx->N, (int)(n * polys * limbs),
                            identity_map((int)limbs), ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_ct_import(hisa_ctx* ctx, const uint64_t* host, uint32_t polys, uint32_t limbs, double scale,
                              hisa_ct** out) {
    return hisa_ct_import_batch(ctx, host, 1, polys, limbs, scale, out);
}

extern "C" int hisa_ct_random_batch(hisa_ctx* ctx, size_t n, uint32_t limbs, double scale, uint64_t counter, hisa_ct** out) {
    if (!ctx || !out || n == 0 || limbs < 1 || limbs > ctx->L) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(alloc_ct_batch(ctx, n, 2, limbs, scale, out));
    // every (ciphertext, polynomial) pair is one batch entry with its own stream counter
    HIP_TRY(ctx, launch_sample_uniform(ctx->d_primes, ctx->prm.seed, 2, counter, identity_map((int)limbs), (int)(n * 2 * limbs),
                                       (u64)limbs * ctx->N, 1, out[0]->data, (int)ctx->log_n, ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_ntt_raw(hisa_ctx* ctx, uint64_t* dev_buf, uint32_t prime_index, size_t n_polys, int inverse) {
    if (!ctx || !dev_buf || prime_index >= ctx->total || n_polys == 0 || n_polys > (1u << 20))
        return fail(ctx, HISA_ERR_ARG, "bad argument");
    PolyMap pm = {};
    pm.period = 1;
    pm.prime_of[0] = (int16_t)prime_index;
    if (inverse) HIP_TRY(ctx, launch_intt(ctx->tabs, (int)ctx->log_n, dev_buf, ctx->N, (int)n_polys, pm, nullptr, ctx->stream));
    else HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, dev_buf, ctx->N, (int)n_polys, pm, ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_key_export(hisa_ctx* ctx, uint64_t key_id, uint64_t* host) {
    if (!ctx || !host) return HISA_ERR_ARG;
    auto it = ctx->keys.find(key_id);
    if (it == ctx->keys.end()) return fail(ctx, HISA_ERR_NO_KEY, "no key %llu", (unsigned long long)key_id);
    const size_t words = (size_t)ctx->dnum * 2 * ctx->total * ctx->N;
    HIP_TRY(ctx, hipMemcpyAsync(host, it->second.data, words * sizeof(u64), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

extern "C" int hisa_secret_export(hisa_ctx* ctx, int64_t* host_coeffs) {
    if (!ctx || !host_coeffs) return HISA_ERR_ARG;
    if (ctx->prm.secret_kind == 1) {
        memcpy(host_coeffs, ctx->sparse_secret.data(), ctx->N * sizeof(i64));
        return HISA_OK;
    }
    Temp raw(ctx, ctx->N * sizeof(i64));
    Temp scratch(ctx, ctx->N * sizeof(u64));
    if (!raw.ok() || !scratch.ok()) return HISA_ERR_OOM;
    PolyMap one = identity_map(1);
    HIP_TRY(ctx, launch_sample_small(ctx->d_primes, ctx->prm.seed, 1, 0, 0, 1, nullptr, 0, one, 1, 0, 0, scratch.u(), raw.as<i64>(),
                                     (int)ctx->log_n, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(host_coeffs, raw.blk->ptr, ctx->N * sizeof(i64), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}
