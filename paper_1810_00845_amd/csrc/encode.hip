// encode / decode in fp64 (the HEAAN-style packing of N/2 complex slots, slot
// j at the root exp(i*pi*5^j/N)), and the centred CRT lift that turns RNS
// coefficients into doubles.  Direct sums with exact integer angle reduction
// into a table of the 2N-th roots of unity.
#include "hisa_internal.hpp"
#include "modarith.hpp"

#define NT 256

// coeffs[p][k] = round( factor * sum_j ( re[p][j] cos(pi e/N) + im[p][j] sin(pi e/N) ) ),  e = g[j] k mod 2N,
// g[j] = 5^(slot of entry j) mod 2N.  One launch encodes n_pts vectors that share the slot list g[count]
// (dense input: g[j] = 5^j; sparse input: only the non-zero slots are listed).
__global__ __launch_bounds__(NT) void encode_kernel(const double* cs, const double* sn, const uint32_t* g, const double* re,
                                                    const double* im, int count, double factor, i64* coeffs, int log_n) {
    const uint32_t k = blockIdx.x * NT + threadIdx.x;
    const uint32_t mask = (2u << log_n) - 1;
    const size_t p = blockIdx.y;
    const double* r = re + p * count;
    const double* m = im ? im + p * count : nullptr;
    double acc = 0.0;
    for (int j = 0; j < count; j++) {
        uint32_t e = (g[j] * k) & mask;
        acc += r[j] * cs[e];
        if (m) acc += m[j] * sn[e];
    }
    coeffs[(p << log_n) + k] = (i64)round(acc * factor);
}

hipError_t launch_encode(const double* cs, const double* sn, const uint32_t* g, const double* re, const double* im,
                         int count, int n_pts, double factor, i64* coeffs, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_pts <= 0) return hipSuccess;
    ProfScope prof__("encode_kernel", st);
    hipLaunchKernelGGL(encode_kernel, dim3((1u << log_n) / NT, n_pts), dim3(NT), 0, st, cs, sn, g, re, im, count, factor,
                       coeffs, log_n);
    return hipGetLastError();
}

// Plaintexts that are piecewise constant -- value v[p][b] on slot set S_b, zero elsewhere -- are linear combinations of
// the nb encodings of the indicator vectors of the S_b: coeffs[p][k] = round(factor * sum_b v[p][b] basis[b][k]) with
// basis[b][k] = sum_{j in S_b} cos(pi g_j k / N), which costs nb terms per coefficient instead of one per slot.
__global__ __launch_bounds__(NT) void encode_basis_kernel(const double* cs, const uint32_t* g, const int* set_begin,
                                                          double* basis, int log_n) {
    const uint32_t k = blockIdx.x * NT + threadIdx.x;
    const uint32_t mask = (2u << log_n) - 1;
    const int b = blockIdx.y;
    double acc = 0.0;
    for (int j = set_begin[b]; j < set_begin[b + 1]; j++) acc += cs[(g[j] * k) & mask];
    basis[((size_t)b << log_n) + k] = acc;
}

__global__ __launch_bounds__(NT) void encode_combine_kernel(const double* basis, int nb, const double* v, double factor,
                                                            i64* coeffs, int log_n) {
    const uint32_t k = blockIdx.x * NT + threadIdx.x;
    const size_t p = blockIdx.y;
    double acc = 0.0;
    for (int b = 0; b < nb; b++) acc += v[p * nb + b] * basis[((size_t)b << log_n) + k];
    coeffs[(p << log_n) + k] = (i64)round(acc * factor);
}

hipError_t launch_encode_basis(const double* cs, const uint32_t* g, const int* set_begin, int nb, double* basis, int log_n,
                               hipStream_t st) {
    DRY_RUN_RETURN();
    if (nb <= 0) return hipSuccess;
    ProfScope prof__("encode_basis_kernel", st);
    hipLaunchKernelGGL(encode_basis_kernel, dim3((1u << log_n) / NT, nb), dim3(NT), 0, st, cs, g, set_begin, basis, log_n);
    return hipGetLastError();
}

hipError_t launch_encode_combine(const double* basis, int nb, const double* v, int n_pts, double factor, i64* coeffs,
                                 int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_pts <= 0) return hipSuccess;
    ProfScope prof__("encode_combine_kernel", st);
    hipLaunchKernelGGL(encode_combine_kernel, dim3((1u << log_n) / NT, n_pts), dim3(NT), 0, st, basis, nb, v, factor, coeffs,
                       log_n);
    return hipGetLastError();
}

// Centred mixed-radix digits v_i in (-q_i/2, q_i/2] with x = v_0 + q_0 (v_1 + q_1 (v_2 + ...)), then Horner in fp64.
// Small centred values have zero top digits, so the float result is accurate for them.
__global__ __launch_bounds__(NT) void crt_to_double_kernel(const PrimeConst* primes, const u64* x, int limbs,
                                                           const u64* ginv, const u64* ginv_sh, int L, double inv_scale,
                                                           double* out, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    double val = 0.0, weight = 1.0;
    // digits are produced low to high; accumulate v_i * (q_0...q_{i-1}) in fp64 from the low end would lose the
    // small terms, so keep the digits and run Horner from the top
    i64 dig[HISA_MAX_Q];
    for (int i = 0; i < limbs; i++) {
        const PrimeConst qi = primes[i];
        u64 t = x[(u64)i * n + j];
        for (int m = 0; m < i; m++) {
            i64 vm = dig[m];
            u64 mag = vm < 0 ? (u64)(-vm) : (u64)vm;
            u64 r = barrett128(0, mag, qi.q, qi.r1, qi.r0);
            if (vm < 0) r = negmod(r, qi.q);
            t = submod(t, r, qi.q);
            t = shoup_mul(t, ginv[(u64)m * L + i], ginv_sh[(u64)m * L + i], qi.q);
        }
        dig[i] = t > qi.half ? (i64)t - (i64)qi.q : (i64)t;
    }
    (void)weight;
    for (int i = limbs - 1; i >= 0; i--) val = val * (double)primes[i].q + (double)dig[i];
    out[j] = val * inv_scale;
}

hipError_t launch_crt_to_double(const PrimeConst* primes, const u64* coeff_form, int limbs, const u64* garner_inv,
                                const u64* garner_inv_sh, int L, double inv_scale, double* out, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    ProfScope prof__("crt_to_double_kernel", st);
    hipLaunchKernelGGL(crt_to_double_kernel, dim3((1u << log_n) / NT), dim3(NT), 0, st, primes, coeff_form, limbs,
                       garner_inv, garner_inv_sh, L, inv_scale, out, log_n);
    return hipGetLastError();
}

// z_j = sum_k m_k exp(i*pi*e/N),  e = 5^j k mod 2N.  One workgroup per slot: thread t sums the coefficients
// k = t, t + NT, ..., then the partial sums are added pairwise through LDS (fixed order: reruns give the same bits).
__global__ __launch_bounds__(NT) void decode_kernel(const double* cs, const double* sn, const double* m, int count,
                                                    double* re, double* im, int log_n) {
    __shared__ double sr[NT], si[NT];
    const int j = blockIdx.x;
    if (j >= count) return;
    const uint32_t n = 1u << log_n, mask = 2 * n - 1;
    // 5^j mod 2N by square and multiply
    uint32_t g = 1, base = 5, ex = (uint32_t)j;
    while (ex) {
        if (ex & 1) g = (g * base) & mask;
        base = (base * base) & mask;
        ex >>= 1;
    }
    double ar = 0.0, ai = 0.0;
    for (uint32_t k = threadIdx.x; k < n; k += NT) {
        const uint32_t e = (g * k) & mask;
        const double v = m[k];
        ar += v * cs[e];
        ai += v * sn[e];
    }
    sr[threadIdx.x] = ar; si[threadIdx.x] = ai;
    __syncthreads();
    for (int h = NT / 2; h > 0; h >>= 1) {
        if ((int)threadIdx.x < h) { sr[threadIdx.x] += sr[threadIdx.x + h]; si[threadIdx.x] += si[threadIdx.x + h]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        re[j] = sr[0];
        if (im) im[j] = si[0];
    }
}

hipError_t launch_decode(const double* cs, const double* sn, const double* m, int count, double* re, double* im, int log_n,
                         hipStream_t st) {
    DRY_RUN_RETURN();
    if (count <= 0) return hipSuccess;
    ProfScope prof__("decode_kernel", st);
    hipLaunchKernelGGL(decode_kernel, dim3(count), dim3(NT), 0, st, cs, sn, m, count, re, im, log_n);
    return hipGetLastError();
}
