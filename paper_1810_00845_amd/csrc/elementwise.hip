// Sampling and limb-wise kernels: the counter-based generator with its
// uniform / ternary / discrete-Gaussian samplers, add / sub / mulPlain /
// mulScalar / mulNoRelin, the combine steps of encryption, decryption and key
// generation, and the NTT-form automorphism gather.  All of them stream
// [..][limb][N] arrays once: they are bound by HBM bandwidth.
#include "hisa_internal.hpp"
#include "modarith.hpp"

#define NT 256

// ---- counter-based generator: rnd(seed, kind, ctr, idx) -------------------
__device__ __forceinline__ u64 mix64(u64 x) {
    x ^= x >> 32; x *= 0x6a09e667f3bcc909ULL;
    x ^= x >> 29; x *= 0xbb67ae8584caa73bULL;
    x ^= x >> 32;
    return x;
}
__device__ __forceinline__ u64 stream_key(u64 seed, u64 kind, u64 ctr) {
    return mix64(seed + 0x3c6ef372fe94f82bULL * (((kind << 56) | ctr) + 1));
}
__device__ __forceinline__ u64 rnd_at(u64 key, u64 idx) { return mix64(key + 0x3c6ef372fe94f82bULL * (idx + 1)); }

__global__ __launch_bounds__(NT) void sample_uniform_kernel(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr,
                                                            PolyMap map, u64 batch_stride, u64 ctr_step, u64* out,
                                                            int log_n) {
    const u64 n = (u64)1 << log_n;
    const int p = blockIdx.y, entry = p % map.period, b = p / map.period;
    const int prime = map.prime_of[entry];
    if (prime < 0) return;
    const PrimeConst pc = primes[prime];
    const u64 key = stream_key(seed, kind, ctr + (u64)b * ctr_step);
    u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    u64 w = rnd_at(key, (u64)prime * n + j);
    out[(u64)b * batch_stride + (u64)entry * n + j] = barrett128(0, w, pc.q, pc.r1, pc.r0);
}

hipError_t launch_sample_uniform(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr, const PolyMap& map, int n_polys,
                                 u64 batch_stride, u64 ctr_step, u64* out, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, n_polys);
    ProfScope prof__("sample_uniform_kernel", st);
    hipLaunchKernelGGL(sample_uniform_kernel, grid, dim3(NT), 0, st, primes, seed, kind, ctr, map, batch_stride, ctr_step,
                       out, log_n);
    return hipGetLastError();
}

// One small signed polynomial per batch entry (ternary secret, or Gaussian
// error, or zero), reduced into every mapped limb.  raw (may be null) receives
// the signed coefficients of batch entry 0.  cdt[k] = floor(2^63 * P(|X| <= k)), k < cdt_n, of the context's
// error distribution: the magnitude is the number of entries the word's upper 63 bits reach, the sign its low bit.
__global__ __launch_bounds__(NT) void sample_small_kernel(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr,
                                                          int noise_on, int ternary, const u64* cdt, int cdt_n, PolyMap map,
                                                          u64 batch_stride, u64 ctr_step, u64* out, i64* raw, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int b = blockIdx.y;
    const u64 key = stream_key(seed, kind, ctr + (u64)b * ctr_step);
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 w = rnd_at(key, j);
    i64 v;
    if (ternary) {
        u64 t = w % 3;
        v = t == 0 ? 0 : (t == 1 ? 1 : -1);
    } else if (noise_on) {
        u64 mag_src = w >> 1;
        i64 mag = 0;
        for (int k = 0; k < cdt_n; k++) mag += (mag_src >= cdt[k]);
        v = (w & 1) ? -mag : mag;
    } else {
        v = 0;
    }
    if (raw && b == 0) raw[j] = v;
    for (int e = 0; e < map.period; e++) {
        int prime = map.prime_of[e];
        if (prime < 0) continue;
        u64 q = primes[prime].q;
        out[(u64)b * batch_stride + (u64)e * n + j] = v >= 0 ? (u64)v : q - (u64)(-v);
    }
}

hipError_t launch_sample_small(const PrimeConst* primes, u64 seed, u64 kind, u64 ctr, int noise_on, int ternary,
                               const u64* cdt, int cdt_n, const PolyMap& map, int n_polys, u64 batch_stride, u64 ctr_step,
                               u64* out, i64* raw, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (!ternary && noise_on && (!cdt || cdt_n <= 0)) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, n_polys);  // n_polys = batch entries here
    ProfScope prof__("sample_small_kernel", st);
    hipLaunchKernelGGL(sample_small_kernel, grid, dim3(NT), 0, st, primes, seed, kind, ctr, noise_on, ternary, cdt, cdt_n,
                       map, batch_stride, ctr_step, out, raw, log_n);
    return hipGetLastError();
}

// ---- add / sub --------------------------------------------------------------
// out[b][p][i] = a[b][p][i] (+|-) b[b][p][i] for p < polys_b, copy of a for the rest.
__global__ __launch_bounds__(NT) void addsub_kernel(const PrimeConst* primes, const u64* a, const u64* b, u64* out, int op,
                                                    int limbs, int polys_a, int polys_b, u64 a_bs, u64 b_bs, u64 o_bs,
                                                    int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y % limbs, poly = blockIdx.y / limbs;
    const u64 bi = blockIdx.z;
    const u64 q = primes[limb].q;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 off = ((u64)poly * limbs + limb) * n + j;
    u64 x = a[bi * a_bs + off];
    if (poly < polys_b) {
        u64 y = b[bi * b_bs + off];
        x = op == OP_ADD ? addmod(x, y, q) : submod(x, y, q);
    }
    out[bi * o_bs + off] = x;
}

hipError_t launch_addsub(const PrimeConst* primes, const u64* a, const u64* b, u64* out, int op, int limbs, int polys_a,
                         int polys_b, u64 n_batch, u64 a_bs, u64 b_bs, u64 o_bs, int log_n, hipStream_t st) {
    if (t_analysis) TALLY(add, HISA_OP_ADD, n_batch, limbs);
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, limbs * polys_a, (unsigned)n_batch);
    ProfScope prof__("addsub_kernel", st);
    hipLaunchKernelGGL(addsub_kernel, grid, dim3(NT), 0, st, primes, a, b, out, op, limbs, polys_a, polys_b, a_bs, b_bs,
                       o_bs, log_n);
    return hipGetLastError();
}

struct LimbConsts {
    u64 v[HISA_MAX_PRIMES];
    u64 v_sh[HISA_MAX_PRIMES];
};

// first polynomial +- per-limb constant (a constant polynomial is that constant at every evaluation point)
__global__ __launch_bounds__(NT) void add_const_kernel(const PrimeConst* primes, const u64* a, u64* out, LimbConsts c,
                                                       int op, int limbs, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y % limbs, poly = blockIdx.y / limbs;
    const u64 q = primes[limb].q;
    const u64 off = ((u64)poly * limbs + limb) * n + (u64)blockIdx.x * NT + threadIdx.x;
    u64 x = a[off];
    if (poly == 0) x = op == OP_ADD ? addmod(x, c.v[limb], q) : submod(x, c.v[limb], q);
    out[off] = x;
}

hipError_t launch_add_const(const PrimeConst* primes, const u64* a, u64* out, const u64* consts, int op, int limbs,
                            int polys, int log_n, hipStream_t st) {
    if (t_analysis) TALLY(add, HISA_OP_ADD, (polys + 1) / 2, limbs);
    DRY_RUN_RETURN();
    LimbConsts c = {};
    for (int i = 0; i < limbs; i++) c.v[i] = consts[i];
    dim3 grid((1u << log_n) / NT, limbs * polys);
    ProfScope prof__("add_const_kernel", st);
    hipLaunchKernelGGL(add_const_kernel, grid, dim3(NT), 0, st, primes, a, out, c, op, limbs, log_n);
    return hipGetLastError();
}

// ---- multiply ---------------------------------------------------------------
// batch entry b is multiplied by plaintext b % pt_period (plaintexts [limbs][N], one after the other)
__global__ __launch_bounds__(NT) void mul_plain_kernel(const PrimeConst* primes, const u64* a, const u64* pt, u64* out,
                                                       int limbs, u64 a_bs, u64 o_bs, unsigned pt_period, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y % limbs, poly = blockIdx.y / limbs;
    const u64 bi = blockIdx.z;
    const PrimeConst pc = primes[limb];
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 off = ((u64)poly * limbs + limb) * n + j;
    const u64* p = pt + (bi % pt_period) * (u64)limbs * n;
    out[bi * o_bs + off] = mulmod_barrett(a[bi * a_bs + off], p[(u64)limb * n + j], pc.q, pc.r1, pc.r0);
}

hipError_t launch_mul_plain(const PrimeConst* primes, const u64* a, const u64* pt, u64* out, int limbs, int polys,
                            u64 n_batch, u64 a_bs, u64 o_bs, int log_n, hipStream_t st, unsigned pt_period) {
    if (t_analysis) TALLY(mul_plain, HISA_OP_MUL_PLAIN, n_batch, limbs);
    DRY_RUN_RETURN();
    if (pt_period == 0 || n_batch == 0 || n_batch > 65535) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, limbs * polys, (unsigned)n_batch);
    ProfScope prof__("mul_plain_kernel", st);
    hipLaunchKernelGGL(mul_plain_kernel, grid, dim3(NT), 0, st, primes, a, pt, out, limbs, a_bs, o_bs, pt_period, log_n);
    return hipGetLastError();
}

__global__ __launch_bounds__(NT) void mul_const_kernel(const PrimeConst* primes, const u64* a, u64* out, LimbConsts c,
                                                       int limbs, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y % limbs;
    const u64 q = primes[limb].q;
    const u64 off = (u64)blockIdx.y * n + (u64)blockIdx.x * NT + threadIdx.x;
    out[off] = shoup_mul(a[off], c.v[limb], c.v_sh[limb], q);
}

hipError_t launch_mul_const(const PrimeConst* primes, const u64* a, u64* out, const u64* consts, int limbs, int polys,
                            int log_n, hipStream_t st) {
    if (t_analysis) TALLY(mul_scalar, HISA_OP_MUL_SCALAR, (polys + 1) / 2, limbs);
    DRY_RUN_RETURN();
    // consts: [limbs] values followed by [limbs] Shoup companions
    LimbConsts c = {};
    for (int i = 0; i < limbs; i++) { c.v[i] = consts[i]; c.v_sh[i] = consts[limbs + i]; }
    dim3 grid((1u << log_n) / NT, limbs * polys);
    ProfScope prof__("mul_const_kernel", st);
    hipLaunchKernelGGL(mul_const_kernel, grid, dim3(NT), 0, st, primes, a, out, c, limbs, log_n);
    return hipGetLastError();
}

// (a0, a1) x (b0, b1) -> (a0 b0, a0 b1 + a1 b0, a1 b1)
__global__ __launch_bounds__(NT) void mul_no_relin_kernel(const PrimeConst* primes, const u64* a, const u64* b, u64* out,
                                                          int limbs, u64 a_bs, u64 b_bs, u64 o_bs, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y;
    const u64 bi = blockIdx.z;
    const PrimeConst pc = primes[limb];
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 o0 = (u64)limb * n + j, o1 = ((u64)limbs + limb) * n + j, o2 = ((u64)2 * limbs + limb) * n + j;
    const u64 a0 = a[bi * a_bs + o0], a1 = a[bi * a_bs + o1];
    const u64 b0 = b[bi * b_bs + o0], b1 = b[bi * b_bs + o1];
    out[bi * o_bs + o0] = mulmod_barrett(a0, b0, pc.q, pc.r1, pc.r0);
    Acc128 acc = {0, 0};
    acc_mad(acc, a0, b1);
    acc_mad(acc, a1, b0);
    out[bi * o_bs + o1] = acc_reduce(acc, pc.q, pc.r1, pc.r0);
    out[bi * o_bs + o2] = mulmod_barrett(a1, b1, pc.q, pc.r1, pc.r0);
}

hipError_t launch_mul_no_relin(const PrimeConst* primes, const u64* a, const u64* b, u64* out, int limbs, u64 n_batch,
                               u64 a_bs, u64 b_bs, u64 o_bs, int log_n, hipStream_t st) {
    if (t_analysis) TALLY(mul, HISA_OP_MUL, n_batch, limbs);
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, limbs, (unsigned)n_batch);
    ProfScope prof__("mul_no_relin_kernel", st);
    hipLaunchKernelGGL(mul_no_relin_kernel, grid, dim3(NT), 0, st, primes, a, b, out, limbs, a_bs, b_bs, o_bs, log_n);
    return hipGetLastError();
}

// ---- encryption profile -----------------------------------------------------
// ct[b] = (-a*s + e + m, a): a already sits in ct[b][1] (NTT form), e[b][limbs][N] in NTT form
__global__ __launch_bounds__(NT) void encrypt_combine_kernel(const PrimeConst* primes, const u64* secret, const u64* pt,
                                                             const u64* e, u64* ct, int limbs, u64 pt_bs, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y;
    const u64 bi = blockIdx.z;
    const PrimeConst pc = primes[limb];
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 off = (u64)limb * n + j;
    u64* c = ct + bi * 2 * limbs * n;
    u64 as = mulmod_barrett(c[(u64)limbs * n + off], secret[off], pc.q, pc.r1, pc.r0);
    u64 v = addmod(negmod(as, pc.q), e[bi * limbs * n + off], pc.q);
    c[off] = addmod(v, pt[bi * pt_bs + off], pc.q);
}

hipError_t launch_encrypt_combine(const PrimeConst* primes, const u64* secret, const u64* pt, const u64* e, u64* ct,
                                  int limbs, u64 n_batch, u64 pt_bs, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, limbs, (unsigned)n_batch);
    ProfScope prof__("encrypt_combine_kernel", st);
    hipLaunchKernelGGL(encrypt_combine_kernel, grid, dim3(NT), 0, st, primes, secret, pt, e, ct, limbs, pt_bs, log_n);
    return hipGetLastError();
}

// pt = c0 + c1*s (+ c2*s^2)
__global__ __launch_bounds__(NT) void decrypt_kernel(const PrimeConst* primes, const u64* secret, const u64* ct, u64* pt,
                                                     int limbs, int polys, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y;
    const PrimeConst pc = primes[limb];
    const u64 off = (u64)limb * n + (u64)blockIdx.x * NT + threadIdx.x;
    const u64 s = secret[off];
    u64 acc = ct[off], sp = s;
    for (int p = 1; p < polys; p++) {
        acc = addmod(acc, mulmod_barrett(ct[(u64)p * limbs * n + off], sp, pc.q, pc.r1, pc.r0), pc.q);
        sp = mulmod_barrett(sp, s, pc.q, pc.r1, pc.r0);
    }
    pt[off] = acc;
}

hipError_t launch_decrypt(const PrimeConst* primes, const u64* secret, const u64* ct, u64* pt, int limbs, int polys,
                          int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, limbs);
    ProfScope prof__("decrypt_kernel", st);
    hipLaunchKernelGGL(decrypt_kernel, grid, dim3(NT), 0, st, primes, secret, ct, pt, limbs, polys, log_n);
    return hipGetLastError();
}

// key digit: b = -a*s + e + [prime in digit] * (P mod q) * target ; a already in key_digit[1]
__global__ __launch_bounds__(NT) void key_combine_kernel(const PrimeConst* primes, const u64* secret, const u64* target,
                                                         const u64* e, const u64* pmod_all, u64* key_digit, int total,
                                                         int L, int alpha, int digit, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int prime = blockIdx.y;
    const PrimeConst pc = primes[prime];
    const u64 off = (u64)prime * n + (u64)blockIdx.x * NT + threadIdx.x;
    u64 a = key_digit[(u64)total * n + off];
    u64 v = addmod(negmod(mulmod_barrett(a, secret[off], pc.q, pc.r1, pc.r0), pc.q), e[off], pc.q);
    if (prime < L && prime / alpha == digit)
        v = addmod(v, mulmod_barrett(pmod_all[prime], target[off], pc.q, pc.r1, pc.r0), pc.q);
    key_digit[off] = v;
}

hipError_t launch_key_combine(const PrimeConst* primes, const u64* secret, const u64* target, const u64* e,
                              const u64* pmod_all, u64* key_digit, int total, int L, int alpha, int digit, int log_n,
                              hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, total);
    ProfScope prof__("key_combine_kernel", st);
    hipLaunchKernelGGL(key_combine_kernel, grid, dim3(NT), 0, st, primes, secret, target, e, pmod_all, key_digit, total, L,
                       alpha, digit, log_n);
    return hipGetLastError();
}

__global__ __launch_bounds__(NT) void square_kernel(const PrimeConst* primes, const u64* s, u64* out, int log_n) {
    const u64 n = (u64)1 << log_n;
    const PrimeConst pc = primes[blockIdx.y];
    const u64 off = (u64)blockIdx.y * n + (u64)blockIdx.x * NT + threadIdx.x;
    out[off] = mulmod_barrett(s[off], s[off], pc.q, pc.r1, pc.r0);
}

hipError_t launch_pointwise_square(const PrimeConst* primes, const u64* s, u64* out, int total, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, total);
    ProfScope prof__("square_kernel", st);
    hipLaunchKernelGGL(square_kernel, grid, dim3(NT), 0, st, primes, s, out, log_n);
    return hipGetLastError();
}

// sigma_g in NTT form is a pure gather: out[i] = in[src(i)] with
// 2*bitrev(src)+1 = (2*bitrev(i)+1)*g mod 2N.  Aligned blocks map to aligned blocks.
__global__ __launch_bounds__(NT) void automorph_ntt_kernel(const u64* in, u64 in_bs, u64* out, u64 out_bs, u64 g,
                                                           int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t i = blockIdx.x * NT + threadIdx.x;
    const uint32_t mask = (2u << log_n) - 1;
    uint32_t e = 2 * (__brev(i) >> (32 - log_n)) + 1;
    uint32_t e2 = (uint32_t)((u64)e * g) & mask;
    uint32_t src = __brev((e2 - 1) >> 1) >> (32 - log_n);
    out[(u64)blockIdx.z * out_bs + (u64)blockIdx.y * n + i] = in[(u64)blockIdx.z * in_bs + (u64)blockIdx.y * n + src];
}

hipError_t launch_automorph_ntt(const u64* in, u64 in_bs, u64* out, u64 out_bs, u64 galois, int n_polys, u64 n_batch,
                                int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, n_polys, (unsigned)n_batch);
    ProfScope prof__("automorph_ntt_kernel", st);
    hipLaunchKernelGGL(automorph_ntt_kernel, grid, dim3(NT), 0, st, in, in_bs, out, out_bs, galois, log_n);
    return hipGetLastError();
}

// The same gather for several automorphisms of the same n_batch inputs in one launch: blockIdx.z = s * n_batch + b,
// out entry (s, b) = sigma_{g[s]}(in entry b).
__global__ __launch_bounds__(NT) void automorph_steps_kernel(const u64* in, u64 in_bs, u64* out, u64 out_bs, GaloisTab tab,
                                                             unsigned n_batch, int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t i = blockIdx.x * NT + threadIdx.x;
    const uint32_t mask = (2u << log_n) - 1;
    const unsigned s = blockIdx.z / n_batch, b = blockIdx.z % n_batch;
    uint32_t e = 2 * (__brev(i) >> (32 - log_n)) + 1;
    uint32_t e2 = (uint32_t)((u64)e * tab.g[s]) & mask;
    uint32_t src = __brev((e2 - 1) >> 1) >> (32 - log_n);
    out[(u64)blockIdx.z * out_bs + (u64)blockIdx.y * n + i] = in[(u64)b * in_bs + (u64)blockIdx.y * n + src];
}

hipError_t launch_automorph_steps(const u64* in, u64 in_bs, u64* out, u64 out_bs, const GaloisTab& tab, int n_steps,
                                  int n_polys, u64 n_batch, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_steps < 1 || n_steps > GALOIS_TAB_MAX || n_batch == 0 || (u64)n_steps * n_batch > 65535) return hipErrorInvalidValue;
    for (int s = 0; s < n_steps; s++)
        if (tab.g[s] == 0) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, n_polys, (unsigned)(n_steps * n_batch));
    ProfScope prof__("automorph_steps_kernel", st);
    hipLaunchKernelGGL(automorph_steps_kernel, grid, dim3(NT), 0, st, in, in_bs, out, out_bs, tab, (unsigned)n_batch, log_n);
    return hipGetLastError();
}

// The part of a sum of rotated ciphertexts that needs no key: out[b] = (plain[b].c0 + sum_s sigma_{g[s]}(rot[s][b].c0),
// plain[b].c1), rot entries ordered rotation-major -- or, with shared_input, entry b for every s --; plain may be null
// (zeros).  Canonical residues in and out.
__global__ __launch_bounds__(NT) void automorph_sum_kernel(const PrimeConst* primes, const u64* rot, u64 rot_bs, int n_rot,
                                                           GaloisTab tab, const u64* plain, u64 plain_bs, u64* out, u64 out_bs,
                                                           unsigned n_batch, int shared_input, int l, int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t i = blockIdx.x * NT + threadIdx.x;
    const uint32_t mask = (2u << log_n) - 1;
    const int limb = blockIdx.y;
    const unsigned b = blockIdx.z;
    const u64 q = primes[limb].q;
    const uint32_t e = 2 * (__brev(i) >> (32 - log_n)) + 1;
    u64 acc = plain ? plain[(u64)b * plain_bs + (u64)limb * n + i] : 0;
    for (int s = 0; s < n_rot; s++) {
        const uint32_t e2 = (uint32_t)((u64)e * tab.g[s]) & mask;
        const uint32_t src = __brev((e2 - 1) >> 1) >> (32 - log_n);
        acc = addmod(acc, rot[((shared_input ? 0 : (u64)s * n_batch) + b) * rot_bs + (u64)limb * n + src], q);
    }
    out[(u64)b * out_bs + (u64)limb * n + i] = acc;
    out[(u64)b * out_bs + (u64)(l + limb) * n + i] = plain ? plain[(u64)b * plain_bs + (u64)(l + limb) * n + i] : 0;
}

hipError_t launch_automorph_sum(const PrimeConst* primes, const u64* rot, u64 rot_bs, int n_rot, const GaloisTab& tab,
                                const u64* plain, u64 plain_bs, u64* out, u64 out_bs, u64 n_batch, int shared_input, int l,
                                int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    const u64 n = (u64)1 << log_n;
    if (!primes || !rot || !out || n_rot < 1 || n_rot > GALOIS_TAB_MAX || n_batch == 0 || n_batch > 65535 || l < 1)
        return hipErrorInvalidValue;
    if (rot_bs < (u64)l * n || out_bs < (u64)2 * l * n || (plain && plain_bs < (u64)2 * l * n)) return hipErrorInvalidValue;
    for (int s = 0; s < n_rot; s++)
        if (tab.g[s] == 0) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, l, (unsigned)n_batch);
    ProfScope prof__("automorph_sum_kernel", st);
    hipLaunchKernelGGL(automorph_sum_kernel, grid, dim3(NT), 0, st, primes, rot, rot_bs, n_rot, tab, plain, plain_bs, out, out_bs,
                       (unsigned)n_batch, shared_input, l, log_n);
    return hipGetLastError();
}

// acc[b][poly] += P * add[b][poly] on the limbs of q_0 .. q_{l-1}, for the polynomials the addend has: what a
// ciphertext contributes to key-switch accumulators that are divided by P later.  acc entries are (ciphertext,
// polynomial) pairs acc_bs words apart; pmod[i] = P mod q_i.
__global__ __launch_bounds__(NT) void fold_addend_kernel(const PrimeConst* primes, u64* acc, u64 acc_bs, const u64* add, u64 add_bs,
                                                         u64 add_ps, int add_polys, const u64* pmod, int log_n) {
    const u64 n = (u64)1 << log_n;
    const int limb = blockIdx.y;
    const u64 e = blockIdx.z, ct = e >> 1;
    const int poly = (int)(e & 1);
    if (poly >= add_polys) return;
    const PrimeConst pc = primes[limb];
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    u64* dst = acc + e * acc_bs + (u64)limb * n + j;
    const u64 v = add[ct * add_bs + (u64)poly * add_ps + (u64)limb * n + j];
    *dst = addmod(*dst, mulmod_barrett(v, pmod[limb], pc.q, pc.r1, pc.r0), pc.q);
}

hipError_t launch_fold_addend(const PrimeConst* primes, u64* acc, u64 acc_bs, const u64* add, u64 add_bs, u64 add_ps,
                              int add_polys, const u64* pmod, u64 n_cts, int l, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    const u64 n = (u64)1 << log_n;
    if (!primes || !acc || !add || !pmod || n_cts == 0 || 2 * n_cts > 65535 || l < 1 || add_polys < 1 || add_polys > 2)
        return hipErrorInvalidValue;
    if (acc_bs < (u64)l * n || add_ps < (u64)l * n || add_bs < (u64)add_polys * l * n) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, l, (unsigned)(2 * n_cts));
    ProfScope prof__("fold_addend_kernel", st);
    hipLaunchKernelGGL(fold_addend_kernel, grid, dim3(NT), 0, st, primes, acc, acc_bs, add, add_bs, add_ps, add_polys, pmod, log_n);
    return hipGetLastError();
}

// signed integer coefficients [n_pts][N] -> residues modulo primes[0..limbs-1] at out[p][0..limbs-1][N], the entries of
// out being out_limbs limbs apart
__global__ __launch_bounds__(NT) void reduce_i64_kernel(const PrimeConst* primes, const i64* coeffs, u64* out, int out_limbs,
                                                        int log_n) {
    const u64 n = (u64)1 << log_n;
    const PrimeConst pc = primes[blockIdx.y];
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const u64 p = blockIdx.z;
    i64 v = coeffs[p * n + j];
    u64 mag = v < 0 ? (u64)0 - (u64)v : (u64)v;
    u64 r = barrett128(0, mag, pc.q, pc.r1, pc.r0);
    out[(p * out_limbs + blockIdx.y) * n + j] = v < 0 ? negmod(r, pc.q) : r;
}

hipError_t launch_reduce_i64(const PrimeConst* primes, const i64* coeffs, u64* out, int limbs, int n_pts, int log_n,
                             hipStream_t st) {
    return launch_reduce_i64(primes, coeffs, out, limbs, limbs, n_pts, log_n, st);
}

hipError_t launch_reduce_i64(const PrimeConst* primes, const i64* coeffs, u64* out, int limbs, int out_limbs, int n_pts,
                             int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_pts <= 0 || limbs <= 0) return hipSuccess;
    dim3 grid((1u << log_n) / NT, limbs, n_pts);
    ProfScope prof__("reduce_i64_kernel", st);
    hipLaunchKernelGGL(reduce_i64_kernel, grid, dim3(NT), 0, st, primes, coeffs, out, out_limbs, log_n);
    return hipGetLastError();
}
