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

// ---------------------------------------------------------------------------
// The same two maps in O(N log N): the "special" FFT over the slot order 5^j
// ---------------------------------------------------------------------------
// With u_k = m_k + i m_{k+n} (n = N/2) the slot values are z_j = sum_{k<n} u_k zeta_j^k, zeta_j = exp(i pi 5^j / N).
// Splitting k into even and odd halves the problem: zeta_j^2 are the slot roots of the ring of half the degree,
// zeta_{j+n/2} = -zeta_j (5^(n/2) = N + 1 mod 2N), so
//     z_j = E_j + zeta_j O_j,   z_{j+n/2} = E_j - zeta_j O_j   (j < n/2),
// a radix-2 decimation-in-time transform from bit-reversed input whose stage of length `len` uses the twiddles
// exp(i pi (5^j mod 4 len) / (2 len)), j < len/2, read from the table of 2N-th roots.  The matrix (zeta_j^k) is
// unitary up to the factor n, so the inverse (encode) runs the stages backwards with conjugate twiddles.
// Stages up to SF_C points run in LDS (one workgroup per chunk of SF_C consecutive points), longer ones one launch each.
#define SF_C 1024
#define SF_LOGC 10
#define SF_T 256
typedef double2 cplx;

__device__ __forceinline__ cplx sf_twiddle(const double* cs, const double* sn, const uint32_t* pow5, uint32_t j, uint32_t len,
                                           int log_n) {
    const uint32_t e = (pow5[j] & (4 * len - 1)) * ((1u << log_n) / (2 * len));
    return make_double2(cs[e], sn[e]);
}
__device__ __forceinline__ cplx sf_mul(cplx a, cplx b) { return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }
__device__ __forceinline__ cplx sf_mulc(cplx a, cplx b) { return make_double2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y); }   // a * conj(b)

// decode direction, stages 2 .. min(n, SF_C): work[vec][pos] from the coefficients m[vec][N]
__global__ __launch_bounds__(SF_T) void sfft_fwd_local_kernel(const double* cs, const double* sn, const uint32_t* pow5,
                                                              const double* m, cplx* work, int log_n) {
    __shared__ cplx buf[SF_C];
    const uint32_t n = 1u << (log_n - 1);
    const uint32_t C = n < SF_C ? n : SF_C;
    const size_t vec = blockIdx.y;
    const uint32_t base = blockIdx.x * C;
    const double* mv = m + (vec << log_n);
    for (uint32_t r = threadIdx.x; r < C; r += SF_T) {
        const uint32_t src = __brev(base + r) >> (32 - (log_n - 1));
        buf[r] = make_double2(mv[src], mv[src + n]);
    }
    __syncthreads();
    for (uint32_t len = 2; len <= C; len <<= 1) {
        const uint32_t half = len >> 1;
        for (uint32_t q = threadIdx.x; q < C / 2; q += SF_T) {
            const uint32_t j = q & (half - 1), i0 = ((q - j) << 1) + j;
            const cplx w = sf_twiddle(cs, sn, pow5, j, len, log_n);
            const cplx u = buf[i0], v = sf_mul(buf[i0 + half], w);
            buf[i0] = make_double2(u.x + v.x, u.y + v.y);
            buf[i0 + half] = make_double2(u.x - v.x, u.y - v.y);
        }
        __syncthreads();
    }
    cplx* wv = work + vec * n + base;
    for (uint32_t r = threadIdx.x; r < C; r += SF_T) wv[r] = buf[r];
}

// one stage of length len > SF_C over work[vec][n], in place; INVERSE: (a, b) -> (a + b, (a - b) conj(w))
template <bool INVERSE>
__global__ __launch_bounds__(SF_T) void sfft_stage_kernel(const double* cs, const double* sn, const uint32_t* pow5, cplx* work,
                                                          uint32_t len, int log_n) {
    const uint32_t n = 1u << (log_n - 1), half = len >> 1;
    const uint32_t q = blockIdx.x * SF_T + threadIdx.x;
    if (q >= n / 2) return;
    cplx* wv = work + (size_t)blockIdx.y * n;
    const uint32_t j = q & (half - 1), i0 = ((q - j) << 1) + j;
    const cplx w = sf_twiddle(cs, sn, pow5, j, len, log_n);
    const cplx a = wv[i0], b = wv[i0 + half];
    if (INVERSE) {
        wv[i0] = make_double2(a.x + b.x, a.y + b.y);
        wv[i0 + half] = sf_mulc(make_double2(a.x - b.x, a.y - b.y), w);
    } else {
        const cplx v = sf_mul(b, w);
        wv[i0] = make_double2(a.x + v.x, a.y + v.y);
        wv[i0 + half] = make_double2(a.x - v.x, a.y - v.y);
    }
}

__global__ __launch_bounds__(SF_T) void sfft_take_kernel(const cplx* work, int count, double* re, double* im, int log_n) {
    const int j = blockIdx.x * SF_T + threadIdx.x;
    if (j >= count) return;
    const cplx z = work[j];
    re[j] = z.x;
    if (im) im[j] = z.y;
}

// encode direction, input: work[vec][slot] = the slot values (zero where there is none): dense rows re/im[vec][count] at
// slots 0 .. count-1, or (slots != null) count values per vector at the listed slots
__global__ __launch_bounds__(SF_T) void sfft_fill_kernel(const double* re, const double* im, const uint32_t* slots, int count,
                                                         cplx* work, int log_n) {
    const uint32_t n = 1u << (log_n - 1);
    const size_t vec = blockIdx.y;
    cplx* wv = work + vec * n;
    if (!slots) {
        const uint32_t j = blockIdx.x * SF_T + threadIdx.x;
        if (j < n) wv[j] = (int)j < count ? make_double2(re[vec * count + j], im ? im[vec * count + j] : 0.0) : make_double2(0.0, 0.0);
    } else {
        // the rows were cleared by the launcher; every listed slot is written once
        const int i = blockIdx.x * SF_T + threadIdx.x;
        if (i < count) wv[slots[i]] = make_double2(re[vec * count + i], im ? im[vec * count + i] : 0.0);
    }
}

// encode direction, stages min(n, SF_C) .. 2, then coefficients k and k + n of the bit-reversed position, rounded
__global__ __launch_bounds__(SF_T) void sfft_inv_local_kernel(const double* cs, const double* sn, const uint32_t* pow5,
                                                              const cplx* work, double factor, i64* coeffs, int log_n) {
    __shared__ cplx buf[SF_C];
    const uint32_t n = 1u << (log_n - 1);
    const uint32_t C = n < SF_C ? n : SF_C;
    const size_t vec = blockIdx.y;
    const uint32_t base = blockIdx.x * C;
    const cplx* wv = work + vec * n + base;
    for (uint32_t r = threadIdx.x; r < C; r += SF_T) buf[r] = wv[r];
    __syncthreads();
    for (uint32_t len = C; len >= 2; len >>= 1) {
        const uint32_t half = len >> 1;
        for (uint32_t q = threadIdx.x; q < C / 2; q += SF_T) {
            const uint32_t j = q & (half - 1), i0 = ((q - j) << 1) + j;
            const cplx w = sf_twiddle(cs, sn, pow5, j, len, log_n);
            const cplx a = buf[i0], b = buf[i0 + half];
            buf[i0] = make_double2(a.x + b.x, a.y + b.y);
            buf[i0 + half] = sf_mulc(make_double2(a.x - b.x, a.y - b.y), w);
        }
        __syncthreads();
    }
    i64* cv = coeffs + (vec << log_n);
    for (uint32_t r = threadIdx.x; r < C; r += SF_T) {
        const uint32_t k = __brev(base + r) >> (32 - (log_n - 1));
        cv[k] = (i64)round(buf[r].x * factor);
        cv[k + n] = (i64)round(buf[r].y * factor);
    }
}

// m[N] -> re/im[count]; work: n complex numbers
hipError_t launch_decode_fft(const double* cs, const double* sn, const uint32_t* pow5, const double* m, int count, void* work,
                             double* re, double* im, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (count <= 0) return hipSuccess;
    if (!cs || !sn || !pow5 || !m || !work || !re || log_n < 2 || log_n > 17 || count > (1 << (log_n - 1))) return hipErrorInvalidValue;
    const uint32_t n = 1u << (log_n - 1), C = n < SF_C ? n : SF_C;
    ProfScope prof__("decode_fft", st);
    hipLaunchKernelGGL(sfft_fwd_local_kernel, dim3(n / C, 1), dim3(SF_T), 0, st, cs, sn, pow5, m, (cplx*)work, log_n);
    for (uint32_t len = 2 * C; len <= n && len > C; len <<= 1)
        hipLaunchKernelGGL(sfft_stage_kernel<false>, dim3((n / 2 + SF_T - 1) / SF_T, 1), dim3(SF_T), 0, st, cs, sn, pow5, (cplx*)work, len, log_n);
    hipLaunchKernelGGL(sfft_take_kernel, dim3((count + SF_T - 1) / SF_T), dim3(SF_T), 0, st, (const cplx*)work, count, re, im, log_n);
    return hipGetLastError();
}

// n_pts slot vectors -> coeffs[n_pts][N] = round(factor * (inverse transform)); values re/im[n_pts][count] at slots
// 0 .. count-1 (slots null) or at slots[count] (device); work: n_pts * n complex numbers
hipError_t launch_encode_fft(const double* cs, const double* sn, const uint32_t* pow5, const double* re, const double* im,
                             const uint32_t* slots, int count, int n_pts, double factor, void* work, i64* coeffs, int log_n,
                             hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_pts <= 0) return hipSuccess;
    if (!cs || !sn || !pow5 || (!re && count) || !work || !coeffs || log_n < 2 || log_n > 17 || count < 0 ||
        count > (1 << (log_n - 1)) || n_pts > 65535)
        return hipErrorInvalidValue;
    const uint32_t n = 1u << (log_n - 1), C = n < SF_C ? n : SF_C;
    ProfScope prof__("encode_fft", st);
    if (slots) {
        hipError_t e = hipMemsetAsync(work, 0, (size_t)n_pts * n * sizeof(cplx), st);
        if (e != hipSuccess) return e;
        if (count) hipLaunchKernelGGL(sfft_fill_kernel, dim3((count + SF_T - 1) / SF_T, n_pts), dim3(SF_T), 0, st, re, im, slots, count, (cplx*)work, log_n);
    } else {
        hipLaunchKernelGGL(sfft_fill_kernel, dim3((n + SF_T - 1) / SF_T, n_pts), dim3(SF_T), 0, st, re, im, slots, count, (cplx*)work, log_n);
    }
    for (uint32_t len = n; len > C; len >>= 1)
        hipLaunchKernelGGL(sfft_stage_kernel<true>, dim3((n / 2 + SF_T - 1) / SF_T, n_pts), dim3(SF_T), 0, st, cs, sn, pow5, (cplx*)work, len, log_n);
    hipLaunchKernelGGL(sfft_inv_local_kernel, dim3(n / C, n_pts), dim3(SF_T), 0, st, cs, sn, pow5, (const cplx*)work, factor, coeffs, log_n);
    return hipGetLastError();
}
