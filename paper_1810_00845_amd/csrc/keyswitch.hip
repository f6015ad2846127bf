// Pieces of hybrid key switching and of rescale that are not transforms:
// fast base conversion (ModUp and the conversion inside ModDown), the inner
// product with the switching key, the final ModDown combine, and the two
// element-wise halves of rescale.
#include "hisa_internal.hpp"
#include "modarith.hpp"

#define NT 256

__global__ __launch_bounds__(NT) void base_conv_kernel(const PrimeConst* primes, ConvArgs g, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int tx = blockIdx.y;
    const u64 b = blockIdx.z;
    const int tp = g.tgt_prime[tx];
    const PrimeConst t = primes[tp];
    const u64* y = g.y + b * g.y_bs + (u64)g.src_pos0 * n + j;
    Acc128 acc = {0, 0};
    u64 wraps = 0;
    for (int i = 0; i < g.a; i++) {
        u64 yi = y[(u64)i * n];
        acc_mad(acc, yi, g.hat[(u64)i * g.total + tp]);
        wraps += (yi > primes[g.src_prime0 + i].half);
        if ((i & 7) == 7) { // keep the high word below t
            acc.lo = acc_reduce(acc, t.q, t.r1, t.r0);
            acc.hi = 0;
        }
    }
    // centred digits: every wrapped y_i stands for y_i - c_i, i.e. one D less
    acc_mad(acc, wraps, t.q - g.dmod[tp]);
    g.out[b * g.out_bs + (u64)g.tgt_pos[tx] * n + j] = acc_reduce(acc, t.q, t.r1, t.r0);
}

hipError_t launch_base_conv(const PrimeConst* primes, const ConvArgs& args, u64 n_batch, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (args.n_targets <= 0 || n_batch == 0) return hipSuccess;
    dim3 grid((1u << log_n) / NT, args.n_targets, (unsigned)n_batch);
    ProfScope prof__("base_conv_kernel", st);
    hipLaunchKernelGGL(base_conv_kernel, grid, dim3(NT), 0, st, primes, args, log_n);
    return hipGetLastError();
}

#define IP_BCHUNK 8
__global__ __launch_bounds__(NT) void inner_product_kernel(const PrimeConst* primes, const u64* ext, u64 ext_bs, int digits,
                                                           int l, int K, int L, const u64* key, int total, u64* acc,
                                                           u64 acc_bs, u64 n_batch, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int x = blockIdx.y;
    const int ext_limbs = l + K;
    const int prime = x < l ? x : L + (x - l);
    const PrimeConst pc = primes[prime];
    const u64 b0 = (u64)blockIdx.z * IP_BCHUNK;
    const u64 b1 = b0 + IP_BCHUNK < n_batch ? b0 + IP_BCHUNK : n_batch;
    for (u64 b = b0; b < b1; b++) {
        Acc128 sb = {0, 0}, sa = {0, 0};
        for (int d = 0; d < digits; d++) {
            u64 e = ext[b * ext_bs + ((u64)d * ext_limbs + x) * n + j];
            acc_mad(sb, e, key[(((u64)d * 2 + 0) * total + prime) * n + j]);
            acc_mad(sa, e, key[(((u64)d * 2 + 1) * total + prime) * n + j]);
            if ((d & 7) == 7) {
                sb.lo = acc_reduce(sb, pc.q, pc.r1, pc.r0); sb.hi = 0;
                sa.lo = acc_reduce(sa, pc.q, pc.r1, pc.r0); sa.hi = 0;
            }
        }
        acc[b * acc_bs + (u64)x * n + j] = acc_reduce(sb, pc.q, pc.r1, pc.r0);
        acc[b * acc_bs + ((u64)ext_limbs + x) * n + j] = acc_reduce(sa, pc.q, pc.r1, pc.r0);
    }
}

hipError_t launch_inner_product(const PrimeConst* primes, const u64* ext, u64 ext_bs, int digits, int l, int K, int L,
                                const u64* key, int total, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, l + K, (unsigned)((n_batch + IP_BCHUNK - 1) / IP_BCHUNK));
    ProfScope prof__("inner_product_kernel", st);
    hipLaunchKernelGGL(inner_product_kernel, grid, dim3(NT), 0, st, primes, ext, ext_bs, digits, l, K, L, key, total, acc,
                       acc_bs, n_batch, log_n);
    return hipGetLastError();
}

__global__ __launch_bounds__(NT) void moddown_final_kernel(const PrimeConst* primes, const u64* acc, u64 acc_bs,
                                                           const u64* conv, u64 conv_bs, const u64* pinv,
                                                           const u64* pinv_sh, const u64* add, u64 add_bs, int add_polys,
                                                           u64 galois, u64* out, u64 out_bs, int l, int K, int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t j = blockIdx.x * NT + threadIdx.x;
    const int i = blockIdx.y % l, p = blockIdx.y / l;
    const u64 b = blockIdx.z;
    const u64 q = primes[i].q;
    u64 v = submod(acc[b * acc_bs + ((u64)p * (l + K) + i) * n + j], conv[b * conv_bs + ((u64)p * l + i) * n + j], q);
    v = shoup_mul(v, pinv[i], pinv_sh[i], q);
    if (p < add_polys) {
        uint32_t src = j;
        if (galois) {
            const uint32_t mask = (2u << log_n) - 1;
            uint32_t e = 2 * (__brev(j) >> (32 - log_n)) + 1;
            uint32_t e2 = (uint32_t)((u64)e * galois) & mask;
            src = __brev((e2 - 1) >> 1) >> (32 - log_n);
        }
        v = addmod(v, add[b * add_bs + ((u64)p * l + i) * n + src], q);
    }
    out[b * out_bs + ((u64)p * l + i) * n + j] = v;
}

hipError_t launch_moddown_final(const PrimeConst* primes, const u64* acc, u64 acc_bs, const u64* conv, u64 conv_bs,
                                const u64* pinv, const u64* pinv_sh, const u64* add, u64 add_bs, int add_polys, u64 galois,
                                u64* out, u64 out_bs, int l, int K, u64 n_batch, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, 2 * l, (unsigned)n_batch);
    ProfScope prof__("moddown_final_kernel", st);
    hipLaunchKernelGGL(moddown_final_kernel, grid, dim3(NT), 0, st, primes, acc, acc_bs, conv, conv_bs, pinv, pinv_sh, add,
                       add_bs, add_polys, galois, out, out_bs, l, K, log_n);
    return hipGetLastError();
}

__global__ __launch_bounds__(NT) void copy_limbs_kernel(const u64* src, u64 src_bs, u64* dst, u64 dst_bs, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 off = (u64)blockIdx.y * n + (u64)blockIdx.x * NT + threadIdx.x;
    dst[(u64)blockIdx.z * dst_bs + off] = src[(u64)blockIdx.z * src_bs + off];
}

hipError_t launch_copy_limbs(const u64* src, u64 src_bs, u64* dst, u64 dst_bs, int limbs, u64 n_batch, int log_n,
                             hipStream_t st) {
    DRY_RUN_RETURN();
    if (limbs <= 0 || n_batch == 0) return hipSuccess;
    dim3 grid((1u << log_n) / NT, limbs, (unsigned)n_batch);
    ProfScope prof__("copy_limbs_kernel", st);
    hipLaunchKernelGGL(copy_limbs_kernel, grid, dim3(NT), 0, st, src, src_bs, dst, dst_bs, log_n);
    return hipGetLastError();
}

// last[bp][N] (coefficient form, modulo q_{l-1}) -> r[bp][i][N], i < l-1:
// r = ((x + h) mod q_last) - h reduced modulo q_i, h = floor(q_last / 2)
__global__ __launch_bounds__(NT) void rescale_spread_kernel(const PrimeConst* primes, const u64* last, u64* r, int l,
                                                            int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int i = blockIdx.y;
    const u64 bp = blockIdx.z;
    const PrimeConst ql = primes[l - 1], qi = primes[i];
    u64 v = csub(last[bp * n + j] + ql.half, ql.q);
    u64 vm = barrett128(0, v, qi.q, qi.r1, qi.r0);
    u64 hm = barrett128(0, ql.half, qi.q, qi.r1, qi.r0);
    r[(bp * (l - 1) + i) * n + j] = submod(vm, hm, qi.q);
}

hipError_t launch_rescale_spread(const PrimeConst* primes, const u64* last, u64* r, int l, u64 n_bp, int log_n,
                                 hipStream_t st) {
    DRY_RUN_RETURN();
    dim3 grid((1u << log_n) / NT, l - 1, (unsigned)n_bp);
    ProfScope prof__("rescale_spread_kernel", st);
    hipLaunchKernelGGL(rescale_spread_kernel, grid, dim3(NT), 0, st, primes, last, r, l, log_n);
    return hipGetLastError();
}

struct RescaleConsts {
    u64 v[HISA_MAX_Q], v_sh[HISA_MAX_Q];
};

__global__ __launch_bounds__(NT) void rescale_final_kernel(const PrimeConst* primes, const u64* ct, const u64* r,
                                                           RescaleConsts c, u64* out, int l, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int i = blockIdx.y;
    const u64 bp = blockIdx.z;
    const u64 q = primes[i].q;
    u64 v = submod(ct[(bp * l + i) * n + j], r[(bp * (l - 1) + i) * n + j], q);
    out[(bp * (l - 1) + i) * n + j] = shoup_mul(v, c.v[i], c.v_sh[i], q);
}

hipError_t launch_rescale_final(const PrimeConst* primes, const u64* ct, const u64* r, const u64* qlinv, const u64* qlinv_sh,
                                u64* out, int l, u64 n_bp, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    RescaleConsts c = {};
    for (int i = 0; i < l - 1; i++) { c.v[i] = qlinv[i]; c.v_sh[i] = qlinv_sh[i]; }
    dim3 grid((1u << log_n) / NT, l - 1, (unsigned)n_bp);
    ProfScope prof__("rescale_final_kernel", st);
    hipLaunchKernelGGL(rescale_final_kernel, grid, dim3(NT), 0, st, primes, ct, r, c, out, l, log_n);
    return hipGetLastError();
}
