// Homomorphic tensor kernels of the paper's runtime (Sec. "Runtime":
// CipherTensor metadata for HW- and CHW-tiling, Algorithm 1 and its SAME-padding
// variant, homomorphic matmul without and with replicas, pooling, degree-2
// activation) on top of the batched HISA primitives.  Host code here only orders launches; the multiply-accumulate
// over (input channel, tap) pairs runs in the two kernels below.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <set>

#include "hisa_internal.hpp"
#include "modarith.hpp"
#include "fparith.hpp"

#define NT 256
#define OCB 4
#define MAX_TAPS 256   // rotation amounts per input ciphertext: filter taps (x channel blocks for CHW-tiling)

struct MacArgs {
    const u64* tap_base[MAX_TAPS];  // per tap: [batch*IC][2][l][N]
    int n_taps, IC, OC, l;
    u64 ct_words;                   // 2*l*N
    const u64* w;                   // scalar: residues [T][OC][l]; plain: plaintexts, NTT form
    u64 w_stride_t, w_stride_oc;    // plain: strides in units of l*N words
    u64* out;                       // [batch*OC][polys][l][N]
    // the fp64 kernels only:
    int polys;                      // polynomials per input / output entry: 2 (0 is read as 2) or 1
    int lq, gap;                    // limb i uses prime i for i < lq and prime i + gap beyond (the special primes of a
                                    // key-switch accumulator's l + K limbs); lq = 0: prime i throughout
    u64 w_words;                    // plain: words per plaintext in memory (0: l * N)
    // plain, optional: a second, one-polynomial input per term on the limbs below lq, multiplied by the same plaintext
    // in the same pass (term (t, b, ic) at x2 + t * x2_tap_words + (b * IC + ic) * x2_words), summed into
    // out2[b * OC + oc] (x2_words apart)
    const u64* x2; u64 x2_tap_words, x2_words; u64* out2;
    // plain, optional: the w_count plaintexts in the limb-major form of pack_plain_kernel (w_count = 0: [plaintext][limb]
    // rows of eight-byte words; w_packed bit 0: limb 0 has six-byte residues, bit 1: the limbs after it have)
    u64 w_count; int w_packed;
};

__device__ __forceinline__ int mac_prime(const MacArgs& g, int limb) { return (g.lq && limb >= g.lq) ? limb + g.gap : limb; }
static inline int mac_polys(const MacArgs& g) { return g.polys == 1 ? 1 : 2; }
// host check of every multiply-accumulate launch, part one: an entry (ct_words apart) must hold the polys * l limbs
// the kernel walks over, and the optional second input its lq limbs
static inline bool mac_shape_ok(const MacArgs& g, int log_n) {
    const u64 n = (u64)1 << log_n;
    if (g.l <= 0 || g.IC <= 0 || g.OC <= 0 || (u64)mac_polys(g) * g.l * n > g.ct_words) return false;
    if (g.lq < 0 || g.lq > g.l) return false;
    if (g.x2 && (u64)g.lq * n > g.x2_words) return false;
    return true;
}

// Part two: the words behind every pointer of a launch (from the pointer to the end of its allocation).  Host only:
// beside the pointers of MacArgs it would not fit the kernel argument area.
struct MacExtents {
    u64 tap[MAX_TAPS];
    u64 out, x2, out2;
    u64 w;   // plain, eight-byte rows only; 0: not known (weights that live outside the context's pool)
};

// The last word each buffer is asked for, by the indexing of the kernels below: tap t reads entries 0 .. batch*IC-1
// (ct_words apart) of polys * l limbs; out takes batch*OC such entries; the second input has n_taps blocks
// (x2_tap_words apart) of batch*IC entries (x2_words apart) of lq limbs, out2 batch*OC of them; plaintext
// (T, oc) starts (T * w_stride_t + oc * w_stride_oc) plaintexts in and is read on l limbs.
static const char* mac_extents_fault(const MacArgs& g, const MacExtents& ex, int batch, int log_n) {
    if (batch <= 0 || g.n_taps <= 0 || g.n_taps > MAX_TAPS || !mac_shape_ok(g, log_n)) return "shape";
    const u64 n = (u64)1 << log_n;
    const u64 entry = (u64)mac_polys(g) * g.l * n;
    const u64 in_need = ((u64)batch * g.IC - 1) * g.ct_words + entry;
    for (int t = 0; t < g.n_taps; t++)
        if (in_need > ex.tap[t]) return "input past its allocation";
    if (((u64)batch * g.OC - 1) * g.ct_words + entry > ex.out) return "output past its allocation";
    if (g.x2) {
        const u64 e2 = (u64)g.lq * n;
        if ((u64)(g.n_taps - 1) * g.x2_tap_words + ((u64)batch * g.IC - 1) * g.x2_words + e2 > ex.x2)
            return "second input past its allocation";
        if (!g.out2 || ((u64)batch * g.OC - 1) * g.x2_words + e2 > ex.out2) return "second output past its allocation";
    }
    if (ex.w && !g.w_count) {
        const u64 wl = g.w_words ? g.w_words : (u64)g.l * n;
        const u64 last = ((u64)g.n_taps * g.IC - 1) * g.w_stride_t + (u64)(g.OC - 1) * g.w_stride_oc;
        if (last * wl + (u64)g.l * n > ex.w) return "plaintexts past their allocation";
    }
    return nullptr;
}

// Every pointer of a launch is looked up among the context's live blocks: data that is not in one is an error too.
static hipError_t mac_bounds(hisa_ctx* ctx, const MacArgs& g, int batch, bool plain) {
    if (g.n_taps <= 0 || g.n_taps > MAX_TAPS) return hipErrorInvalidValue;
    MacExtents ex = {};
    for (int t = 0; t < g.n_taps; t++) ex.tap[t] = dev_words_behind(ctx, g.tap_base[t]);
    ex.out = dev_words_behind(ctx, g.out);
    if (g.x2) { ex.x2 = dev_words_behind(ctx, g.x2); ex.out2 = g.out2 ? dev_words_behind(ctx, g.out2) : 0; }
    if (plain && g.w) ex.w = dev_words_behind(ctx, g.w);
    if (const char* why = mac_extents_fault(g, ex, batch, (int)ctx->log_n)) {
        fail(ctx, HISA_ERR_ARG, "multiply-accumulate refused: %s (l %d, lq %d, gap %d, polys %d, IC %d, OC %d, taps %d, batch %d)",
             why, g.l, g.lq, g.gap, mac_polys(g), g.IC, g.OC, g.n_taps, batch);
        return hipErrorInvalidDevicePointer;
    }
    return hipSuccess;
}

// the library's error for a launcher's: a refusal by the checks above keeps its own message
static int mac_fail(hisa_ctx* ctx, hipError_t e, const char* what) {
    if (e == hipErrorInvalidDevicePointer) return HISA_ERR_ARG;
    return fail(ctx, e == hipErrorInvalidValue ? HISA_ERR_ARG : HISA_ERR_HIP, "%s multiply-accumulate: %s", what, hipGetErrorString(e));
}

extern "C" int hisa_check_mac_extents(const hisa_mac_extents* a) {
    if (!a || a->n_taps <= 0 || a->n_taps > MAX_TAPS || a->log_n < 1 || a->log_n > 17) return HISA_ERR_ARG;
    if (a->n_taps > 1 && !a->tap_words) return HISA_ERR_ARG;
    MacArgs g = {};
    MacExtents ex = {};
    g.n_taps = a->n_taps; g.IC = a->ic; g.OC = a->oc; g.l = a->limbs; g.polys = a->polys; g.lq = a->lq; g.gap = a->gap;
    g.ct_words = a->ct_words;
    for (int t = 0; t < a->n_taps; t++) ex.tap[t] = a->tap_words ? a->tap_words[t] : a->tap0_words;
    ex.out = a->out_words;
    if (a->x2_extent || a->out2_extent) {
        g.x2 = (const u64*)8; g.out2 = (u64*)8;   // never dereferenced: only "a second input is present"
        g.x2_tap_words = a->x2_tap_words; g.x2_words = a->x2_words;
        ex.x2 = a->x2_extent; ex.out2 = a->out2_extent;
    }
    g.w_words = a->w_words; g.w_stride_t = a->w_stride_t; g.w_stride_oc = a->w_stride_oc;
    ex.w = a->w_extent;
    return mac_extents_fault(g, ex, a->batch, a->log_n) ? HISA_ERR_ARG : HISA_OK;
}

// out[b][oc] = sum over T = (tap, ic) of  w[T][oc] * x[tap][b][ic]   (integer weights, one per limb)
__global__ __launch_bounds__(NT) void scalar_mac_kernel(const PrimeConst* primes, MacArgs g, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int pl = blockIdx.y, limb = pl % g.l;
    const int ocblocks = (g.OC + OCB - 1) / OCB;
    const int b = blockIdx.z / ocblocks, oc0 = (blockIdx.z % ocblocks) * OCB;
    const PrimeConst pc = primes[limb];
    Acc128 acc[OCB];
    for (int o = 0; o < OCB; o++) acc[o] = {0, 0};
    int pending = 0;
    for (int t = 0; t < g.n_taps; t++) {
        const u64* x = g.tap_base[t] + (u64)b * g.IC * g.ct_words + (u64)pl * n + j;
        const u64* w = g.w + ((u64)t * g.IC * g.OC + oc0) * g.l + limb;
        for (int ic = 0; ic < g.IC; ic++) {
            const u64 xv = x[(u64)ic * g.ct_words];
            for (int o = 0; o < OCB; o++)
                if (oc0 + o < g.OC) acc_mad(acc[o], xv, w[((u64)ic * g.OC + o) * g.l]);
            if (++pending == 8) {  // keep the high words below q
                for (int o = 0; o < OCB; o++) { acc[o].lo = acc_reduce(acc[o], pc.q, pc.r1, pc.r0); acc[o].hi = 0; }
                pending = 0;
            }
        }
    }
    for (int o = 0; o < OCB; o++)
        if (oc0 + o < g.OC)
            g.out[((u64)b * g.OC + oc0 + o) * g.ct_words + (u64)pl * n + j] = acc_reduce(acc[o], pc.q, pc.r1, pc.r0);
}

// The same sum in exact fp64 arithmetic (every prime below 2^50): a modular product is six full-rate instructions
// instead of a 64x64 high/low product pair at quarter rate, and OCF outputs share each load of x.  The weights
// (centred doubles) are the same for every thread and arrive through scalar loads.
// Range: a term is at most 0.7 p in magnitude, eight of them on top of a normalised value stay below 6.1 p < 2^53.
#define OCF 16
#define ICU 4
typedef const __attribute__((address_space(4))) double* mac_cdouble_ptr;
// wf: [l][T][OC] (the OCF weights of one x value are contiguous: wide scalar loads)
__global__ __launch_bounds__(NT) void scalar_mac_fp_kernel(const FpPrime* fprimes, MacArgs g, const double* wf, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int pl = blockIdx.y, limb = pl % g.l;
    const int ocblocks = (g.OC + OCF - 1) / OCF;
    const int b = blockIdx.z / ocblocks, oc0 = (blockIdx.z % ocblocks) * OCF;
    const mac_cdouble_ptr fp = (mac_cdouble_ptr)(unsigned long long)&fprimes[mac_prime(g, limb)].p;
    const double p = fp[0], pinv = fp[1];
    const bool full = oc0 + OCF <= g.OC;     // all OCF outputs exist (uniform over the workgroup)
    double acc[OCF];
#pragma unroll
    for (int o = 0; o < OCF; o++) acc[o] = 0.0;
    int pending = 0;
    for (int t = 0; t < g.n_taps; t++) {
        const u64* x = g.tap_base[t] + (u64)b * g.IC * g.ct_words + (u64)pl * n + j;
        const mac_cdouble_ptr w =
            (mac_cdouble_ptr)(unsigned long long)(wf + ((u64)limb * g.n_taps + t) * g.IC * g.OC + oc0);
        for (int ic0 = 0; ic0 < g.IC; ic0 += ICU) {
            // the loads of ICU input channels first, then their arithmetic
            double xv[ICU];
#pragma unroll
            for (int u = 0; u < ICU; u++) {
                const int ic = ic0 + u < g.IC ? ic0 + u : g.IC - 1;
                xv[u] = fp_from_u64(x[(u64)ic * g.ct_words]);
            }
#pragma unroll
            for (int u = 0; u < ICU; u++) {
                if (ic0 + u < g.IC) {
                    const mac_cdouble_ptr wi = w + (u64)(ic0 + u) * g.OC;
                    if (full) {
#pragma unroll
                        for (int o = 0; o < OCF; o++) acc[o] += fp_mulmod(xv[u], wi[o], p, pinv);
                    } else {
#pragma unroll
                        for (int o = 0; o < OCF; o++)
                            if (oc0 + o < g.OC) acc[o] += fp_mulmod(xv[u], wi[o], p, pinv);
                    }
                }
            }
            pending += ICU;
            if (pending >= 8) {
#pragma unroll
                for (int o = 0; o < OCF; o++) acc[o] = fp_norm(acc[o], p, pinv);
                pending = 0;
            }
        }
    }
#pragma unroll
    for (int o = 0; o < OCF; o++)
        if (oc0 + o < g.OC)
            g.out[((u64)b * g.OC + oc0 + o) * g.ct_words + (u64)pl * n + j] = fp_canonical(acc[o], p, pinv);
}

// out[b][oc] = sum over T = (tap, ic) of  pt[T][oc] (slot-wise) x[tap][b][ic]
__global__ __launch_bounds__(NT) void plain_mac_kernel(const PrimeConst* primes, MacArgs g, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int limb = blockIdx.y;
    const int b = blockIdx.z / g.OC, oc = blockIdx.z % g.OC;
    const PrimeConst pc = primes[limb];
    const u64 ln = (u64)g.l * n;
    Acc128 a0 = {0, 0}, a1 = {0, 0};
    int pending = 0;
    for (int t = 0; t < g.n_taps; t++) {
        const u64* x = g.tap_base[t] + (u64)b * g.IC * g.ct_words + (u64)limb * n + j;
        for (int ic = 0; ic < g.IC; ic++) {
            const u64 T = (u64)t * g.IC + ic;
            const u64 wv = g.w[(T * g.w_stride_t + (u64)oc * g.w_stride_oc) * ln + (u64)limb * n + j];
            acc_mad(a0, x[(u64)ic * g.ct_words], wv);
            acc_mad(a1, x[(u64)ic * g.ct_words + ln], wv);
            if (++pending == 8) {
                a0.lo = acc_reduce(a0, pc.q, pc.r1, pc.r0); a0.hi = 0;
                a1.lo = acc_reduce(a1, pc.q, pc.r1, pc.r0); a1.hi = 0;
                pending = 0;
            }
        }
    }
    u64* o = g.out + ((u64)b * g.OC + oc) * g.ct_words + (u64)limb * n + j;
    o[0] = acc_reduce(a0, pc.q, pc.r1, pc.r0);
    o[ln] = acc_reduce(a1, pc.q, pc.r1, pc.r0);
}

// The same sum on the matrix cores.  Over k = (tap, channel) it is a dense contraction out[oc][e] = sum_k W[k][oc] X[k][e]
// of integers below 2^50 in magnitude.  Both factors are split into signed base-256 digits (DA for the weights: three
// for masked convolutions, whose fixed-point weights are about 20 bits, up to seven; DB = 6 or 7 for the residues,
// by the size of the largest prime); the DA x DB digit-by-digit products are int8 MFMAs accumulating exactly in
// int32, summed per diagonal a + b = s; the value sum_s D_s 256^s is then reduced modulo p in fp64.  Exact, so
// bit-identical to the other two kernels.
//   block: 4 waves; 64 coefficients x 64 outputs; wave w owns outputs 16 w .. 16 w + 15 (rows of the MFMA tile) and
//   four 16-coefficient column tiles; k advances 64 at a time (one 16x16x64 MFMA per digit pair and column tile).
//   The digits of X are staged in LDS as [digit][k / 16][e][k % 16]: a thread converts 16 consecutive k of one
//   coefficient and writes 16 bytes per digit, exactly the operand a lane reads back.  The next 16 words are loaded
//   from global memory before the MFMAs of the current ones.
//   Operand slots: lane l of an operand holds row or column l % 16 and the sixteen k values of group l / 16; both
//   operands use the same k <-> slot assignment, which is all the contraction needs.  Result: lane l, register r
//   holds row 4 (l / 16) + r, column l % 16.
#define MT_E 64
#define MT_OC 64
#define MT_K 64
#define MAC_DIGITS 7   // most digits of either factor
typedef int v4i_t __attribute__((ext_vector_type(4)));

// the seven signed base-256 digits of x (|x| < 2^55) in the low seven bytes: (x + B) ^ B with B = 0x80 in each of them
__host__ __device__ __forceinline__ u64 balanced_digits(u64 x) {
    const u64 B = 0x0080808080808080ULL;
    return (x + B) ^ B;
}

template <int DA, int DB>
__global__ __launch_bounds__(256) void scalar_mac_mfma_kernel(const FpPrime* fprimes, MacArgs g, const int8_t* wd, int K,
                                                              int K_pad, int OC_pad, const double* c3, int log_n) {
    constexpr int MAC_DIAGS = DA + DB - 1;
    __shared__ v4i_t xd[DB][MT_K / 16][MT_E];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const u64 n = (u64)1 << log_n;
    const u64 e0 = (u64)blockIdx.x * MT_E;
    const int pl = blockIdx.y, limb = pl % g.l;
    const int ocblocks = OC_pad / MT_OC;
    const int b = blockIdx.z / ocblocks, oc0 = (blockIdx.z % ocblocks) * MT_OC + wave * 16;

    v4i_t acc[4][MAC_DIAGS];
#pragma unroll
    for (int ct = 0; ct < 4; ct++)
#pragma unroll
        for (int sdiag = 0; sdiag < MAC_DIAGS; sdiag++) acc[ct][sdiag] = (v4i_t){0, 0, 0, 0};

    // the 16 words X[k][e0 + lane], k = kc + 16 wave + s (zero beyond K)
    u64 xs[16];
    auto load_x = [&](int kc) {
        int k = kc + wave * 16;
        int tap = k / g.IC, ic = k - tap * g.IC;
#pragma unroll
        for (int sl = 0; sl < 16; sl++) {
            xs[sl] = 0;
            if (k + sl < K) xs[sl] = g.tap_base[tap][((u64)b * g.IC + ic) * g.ct_words + (u64)pl * n + e0 + lane];
            if (++ic == g.IC) { ic = 0; tap++; }
        }
    };
    // the wave's weight digits of the next 64 k (lane: row lane % 16, k group lane / 16), fetched one step ahead as well
    v4i_t A[DA], An[DA];
    auto load_a = [&](int kc, v4i_t (&dst)[DA]) {
#pragma unroll
        for (int a = 0; a < DA; a++)
            dst[a] = *(const v4i_t*)(wd + (((u64)(limb * MAC_DIGITS + a) * OC_pad + oc0 + (lane & 15)) * K_pad + kc + 16 * (lane >> 4)));
    };
    load_x(0);
    load_a(0, An);
    for (int kc = 0; kc < K_pad; kc += MT_K) {
#pragma unroll
        for (int sl = 0; sl < 16; sl++) xs[sl] = balanced_digits(xs[sl]);
#pragma unroll
        for (int a = 0; a < DB; a++) {
            v4i_t d;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                uint32_t wq = 0;
#pragma unroll
                for (int i = 0; i < 4; i++) wq |= (uint32_t)((xs[4 * q + i] >> (8 * a)) & 0xFF) << (8 * i);
                d[q] = (int)wq;
            }
            xd[a][wave][lane] = d;
        }
        __syncthreads();
#pragma unroll
        for (int a = 0; a < DA; a++) A[a] = An[a];
        if (kc + MT_K < K_pad) { load_x(kc + MT_K); load_a(kc + MT_K, An); }
#pragma unroll
        for (int ct = 0; ct < 4; ct++) {
            v4i_t Bv[DB];
#pragma unroll
            for (int bb = 0; bb < DB; bb++) Bv[bb] = xd[bb][lane >> 4][ct * 16 + (lane & 15)];
#pragma unroll
            for (int a = 0; a < DA; a++)
#pragma unroll
                for (int bb = 0; bb < DB; bb++)
                    acc[ct][a + bb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[a], Bv[bb], acc[ct][a + bb], 0, 0, 0);
        }
        __syncthreads();
    }

    // sum_s D_s 256^s mod p: three diagonals at a time are combined exactly in a double (below 2^48), then five
    // modular products with 2^(24 g) mod p
    const mac_cdouble_ptr fp = (mac_cdouble_ptr)(unsigned long long)&fprimes[mac_prime(g, limb)].p;
    const double p = fp[0], pinv = fp[1];
    const mac_cdouble_ptr cg = (mac_cdouble_ptr)(unsigned long long)(c3 + limb * 5);
#pragma unroll
    for (int ct = 0; ct < 4; ct++) {
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int oc = oc0 + 4 * (lane >> 4) + r;
            double sum = 0.0;
#pragma unroll
            for (int gq = 0; 3 * gq < MAC_DIAGS; gq++) {
                double G = (double)acc[ct][3 * gq][r];
                if (3 * gq + 1 < MAC_DIAGS) G = __builtin_fma((double)acc[ct][3 * gq + 1][r], 256.0, G);
                if (3 * gq + 2 < MAC_DIAGS) G = __builtin_fma((double)acc[ct][3 * gq + 2][r], 65536.0, G);
                sum += fp_mulmod(G, cg[gq], p, pinv);
            }
            if (oc < g.OC)
                g.out[((u64)b * g.OC + oc) * g.ct_words + (u64)pl * n + e0 + ct * 16 + (lane & 15)] = fp_canonical(sum, p, pinv);
        }
    }
}

// The slot-wise sum in exact fp64 arithmetic (every prime below 2^50).  A thread forms OCP outputs (4, or 8 when there
// are at least 8) from each pair of
// ciphertext words it loads (the inputs are re-read once per group of OCP outputs, not once per output), and two
// (tap, channel) terms are loaded before their arithmetic.
#define ICP 2
// WITH_X2: the optional second input is present (a separate instantiation, so that the common form keeps its
// straight-line loads)
template <bool WITH_X2, int OCP>
__device__ __forceinline__ void plain_mac_fp_body(const FpPrime* fprimes, const MacArgs& g, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    // the groups of outputs of one limb are neighbours in launch order (and land on the same XCD: the number of
    // blocks along x is a multiple of 8 from N = 2^11 on), so the ciphertext words they all read stay in that L2
    const int limb = blockIdx.z;
    const int ocblocks = (g.OC + OCP - 1) / OCP;
    const int b = blockIdx.y / ocblocks, oc0 = (blockIdx.y % ocblocks) * OCP;
    const mac_cdouble_ptr fp = (mac_cdouble_ptr)(unsigned long long)&fprimes[mac_prime(g, limb)].p;
    const double p = fp[0], pinv = fp[1];
    const u64 ln = (u64)g.l * n, wl = g.w_words ? g.w_words : ln;
    const bool two = g.polys != 1;      // one-polynomial entries: the second accumulator idles
    const bool third = WITH_X2 && limb < g.lq;
    double a0[OCP], a1[OCP], a2[OCP];
#pragma unroll
    for (int o = 0; o < OCP; o++) a0[o] = a1[o] = a2[o] = 0.0;
    int pending = 0;
    for (int t = 0; t < g.n_taps; t++) {
        const u64* x = g.tap_base[t] + (u64)b * g.IC * g.ct_words + (u64)limb * n + j;
        const u64* w = g.w + ((u64)t * g.IC * g.w_stride_t + (u64)oc0 * g.w_stride_oc) * wl + (u64)limb * n + j;
        const u64* x2 = third ? g.x2 + (u64)t * g.x2_tap_words + (u64)b * g.IC * g.x2_words + (u64)limb * n + j : nullptr;
        for (int ic0 = 0; ic0 < g.IC; ic0 += ICP) {
            u64 xb[ICP], xa[ICP], xc[ICP], wv[ICP][OCP];
#pragma unroll
            for (int u = 0; u < ICP; u++) {
                const int ic = ic0 + u < g.IC ? ic0 + u : g.IC - 1;
                xb[u] = x[(u64)ic * g.ct_words];
                xa[u] = two ? x[(u64)ic * g.ct_words + ln] : 0;
                xc[u] = third ? x2[(u64)ic * g.x2_words] : 0;
#pragma unroll
                for (int o = 0; o < OCP; o++) {
                    const int oo = oc0 + o < g.OC ? o : 0;
                    wv[u][o] = w[((u64)ic * g.w_stride_t + (u64)oo * g.w_stride_oc) * wl];
                }
            }
#pragma unroll
            for (int u = 0; u < ICP; u++) {
                if (ic0 + u < g.IC) {
                    const double fb = fp_from_u64(xb[u]), fa = fp_from_u64(xa[u]), fc = fp_from_u64(xc[u]);
#pragma unroll
                    for (int o = 0; o < OCP; o++) {
                        const double wf = fp_from_u64(wv[u][o]);
                        a0[o] += fp_mulmod(fb, wf, p, pinv);
                        a1[o] += fp_mulmod(fa, wf, p, pinv);
                        if (third) a2[o] += fp_mulmod(fc, wf, p, pinv);
                    }
                }
            }
            pending += ICP;
            if (pending >= 4) {   // canonical operands: a term can reach 0.9 p, four of them on a normalised value 4.1 p
#pragma unroll
                for (int o = 0; o < OCP; o++) {
                    a0[o] = fp_norm(a0[o], p, pinv); a1[o] = fp_norm(a1[o], p, pinv);
                    if (third) a2[o] = fp_norm(a2[o], p, pinv);
                }
                pending = 0;
            }
        }
    }
#pragma unroll
    for (int o = 0; o < OCP; o++) {
        if (oc0 + o < g.OC) {
            u64* dst = g.out + ((u64)b * g.OC + oc0 + o) * g.ct_words + (u64)limb * n + j;
            dst[0] = fp_canonical(a0[o], p, pinv);
            if (two) dst[ln] = fp_canonical(a1[o], p, pinv);
            if (third) g.out2[((u64)b * g.OC + oc0 + o) * g.x2_words + (u64)limb * n + j] = fp_canonical(a2[o], p, pinv);
        }
    }
}

// The plaintexts of a plan: limb-major -- the rows that a group of outputs reads for one term lie side by side -- and
// with six bytes per residue where the prime is below 2^48 (the row layout of pack_plain_kernel), a quarter less of the
// bytes that bound this kernel.  FORM of the rows this block reads: 1 eight-byte residues, 2 six-byte residues (a
// template argument, so that the loads of a term stay one straight line).  Two neighbouring coefficients per thread:
// sixteen-byte loads of the ciphertext words and of eight-byte rows, eight + four bytes of a six-byte row.
// Two-polynomial entries on the primes q_0.. only.
template <int OCP, int FORM>
__device__ __forceinline__ void plain_mac_fp_body2(const FpPrime* fprimes, const MacArgs& g, int log_n) {
    typedef unsigned long long ull2_t __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u64 n = (u64)1 << log_n;
    const u64 j = ((u64)blockIdx.x * NT + threadIdx.x) * 2;
    const int limb = blockIdx.z;
    const int ocblocks = (g.OC + OCP - 1) / OCP;
    const int b = blockIdx.y / ocblocks, oc0 = (blockIdx.y % ocblocks) * OCP;
    const mac_cdouble_ptr fp = (mac_cdouble_ptr)(unsigned long long)&fprimes[limb].p;
    const double p = fp[0], pinv = fp[1];
    const u64 ln = (u64)g.l * n;
    double a0[OCP][2], a1[OCP][2];
#pragma unroll
    for (int o = 0; o < OCP; o++) a0[o][0] = a0[o][1] = a1[o][0] = a1[o][1] = 0.0;
    int pending = 0;
    const u64 lo_off = (j >> 7) * 768 + (j & 127) * 4, hi_off = (j >> 7) * 768 + 512 + (j & 127) * 2;
    const u64 b0 = (g.w_packed & 1) ? 6 : 8, b1 = (g.w_packed & 2) ? 6 : 8, rb = (FORM == 2 ? 6 : 8) * n;
    // term = (tap, input): the loads of the next term are issued before the arithmetic of the current one
    const char* wlimb = (const char*)g.w + (limb ? b0 + (u64)(limb - 1) * b1 : 0) * n * g.w_count + (u64)oc0 * g.w_stride_oc * rb;
    auto load = [&](int t, int ic, ull2_t& xb, ull2_t& xa, ull2_t (&wv)[OCP]) {
        const u64* x = g.tap_base[t] + ((u64)b * g.IC + ic) * g.ct_words + (u64)limb * n + j;
        xb = *(const ull2_t*)x;
        xa = *(const ull2_t*)(x + ln);
        const char* wp = wlimb + ((u64)t * g.IC + ic) * g.w_stride_t * rb;
#pragma unroll
        for (int o = 0; o < OCP; o++) {
            const int oo = oc0 + o < g.OC ? o : 0;
            const char* row = wp + (u64)oo * g.w_stride_oc * rb;
            if (FORM == 2) {
                const u32x2 lo = *(const u32x2*)(row + lo_off);
                const uint32_t hi = *(const uint32_t*)(row + hi_off);
                wv[o].x = (u64)lo.x | ((u64)(hi & 0xFFFFu) << 32);
                wv[o].y = (u64)lo.y | ((u64)(hi >> 16) << 32);
            } else {
                wv[o] = *(const ull2_t*)(row + 8 * j);
            }
        }
    };
    ull2_t xb, xa, wv[OCP], nxb, nxa, nwv[OCP];
    load(0, 0, xb, xa, wv);
    for (int t = 0; t < g.n_taps; t++) {
        for (int ic = 0; ic < g.IC; ic++) {
            const bool more = ic + 1 < g.IC || t + 1 < g.n_taps;
            if (more) load(ic + 1 < g.IC ? t : t + 1, ic + 1 < g.IC ? ic + 1 : 0, nxb, nxa, nwv);
            const double fb[2] = {fp_from_u64(xb.x), fp_from_u64(xb.y)}, fa[2] = {fp_from_u64(xa.x), fp_from_u64(xa.y)};
#pragma unroll
            for (int o = 0; o < OCP; o++) {
                const double wf[2] = {fp_from_u64(wv[o].x), fp_from_u64(wv[o].y)};
#pragma unroll
                for (int c = 0; c < 2; c++) {
                    a0[o][c] += fp_mulmod(fb[c], wf[c], p, pinv);
                    a1[o][c] += fp_mulmod(fa[c], wf[c], p, pinv);
                }
            }
            if (++pending == 4) {   // canonical operands: a term can reach 0.9 p, four of them on a normalised value 4.1 p
#pragma unroll
                for (int o = 0; o < OCP; o++)
#pragma unroll
                    for (int c = 0; c < 2; c++) { a0[o][c] = fp_norm(a0[o][c], p, pinv); a1[o][c] = fp_norm(a1[o][c], p, pinv); }
                pending = 0;
            }
            if (more) {
                xb = nxb; xa = nxa;
#pragma unroll
                for (int o = 0; o < OCP; o++) wv[o] = nwv[o];
            }
        }
    }
#pragma unroll
    for (int o = 0; o < OCP; o++) {
        if (oc0 + o < g.OC) {
            u64* dst = g.out + ((u64)b * g.OC + oc0 + o) * g.ct_words + (u64)limb * n + j;
            ull2_t r0, r1;
            r0.x = fp_canonical(a0[o][0], p, pinv); r0.y = fp_canonical(a0[o][1], p, pinv);
            r1.x = fp_canonical(a1[o][0], p, pinv); r1.y = fp_canonical(a1[o][1], p, pinv);
            *(ull2_t*)dst = r0;
            *(ull2_t*)(dst + ln) = r1;
        }
    }
}

template <bool WITH_X2, int OCP, bool PACKED = false>
__global__ __launch_bounds__(NT) void plain_mac_fp_kernel(const FpPrime* fprimes, MacArgs g, int log_n) {
    if (!PACKED) plain_mac_fp_body<WITH_X2, OCP>(fprimes, g, log_n);
    else if (g.w_packed >> (blockIdx.z ? 1 : 0) & 1) plain_mac_fp_body2<OCP, 2>(fprimes, g, log_n);
    else plain_mac_fp_body2<OCP, 1>(fprimes, g, log_n);
}

// analysis mode: a multiply-accumulate launch stands for one term per (image, output, tap, input)
static void count_mac(const MacArgs& g, int batch, bool plain) {
    if (!t_analysis) return;
    const uint64_t terms = (uint64_t)batch * g.OC * g.n_taps * g.IC;
    if (plain) TALLY(mac_plain, HISA_OP_MAC_PLAIN, terms, g.l);
    else TALLY(mac_scalar, HISA_OP_MAC_SCALAR, terms, g.l);
}

static hipError_t launch_scalar_mac(hisa_ctx* ctx, const PrimeConst* primes, const MacArgs& g, int batch, int log_n, hipStream_t st) {
    count_mac(g, batch, false);
    DRY_RUN_RETURN();
    if (hipError_t be = mac_bounds(ctx, g, batch, false)) return be;
    // the integer kernels know two-polynomial entries on the primes q_0.. only
    if (!primes || !g.w || !g.out || g.n_taps <= 0 || g.n_taps > MAX_TAPS || g.polys == 1 || g.lq || g.x2 || g.w_words ||
        !mac_shape_ok(g, log_n))
        return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, 2 * g.l, batch * ((g.OC + OCB - 1) / OCB));
    ProfScope prof__("scalar_mac_kernel", st);
    hipLaunchKernelGGL(scalar_mac_kernel, grid, dim3(NT), 0, st, primes, g, log_n);
    return hipGetLastError();
}

static hipError_t launch_scalar_mac_fp(hisa_ctx* ctx, const FpPrime* fprimes, const MacArgs& g, const double* wf, int batch, int log_n,
                                       hipStream_t st) {
    count_mac(g, batch, false);
    DRY_RUN_RETURN();
    if (hipError_t be = mac_bounds(ctx, g, batch, false)) return be;
    if (!fprimes || !wf || !g.out || g.n_taps <= 0 || g.n_taps > MAX_TAPS || !mac_shape_ok(g, log_n)) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, mac_polys(g) * g.l, batch * ((g.OC + OCF - 1) / OCF));
    ProfScope prof__("scalar_mac_fp_kernel", st);
    hipLaunchKernelGGL(scalar_mac_fp_kernel, grid, dim3(NT), 0, st, fprimes, g, wf, log_n);
    return hipGetLastError();
}

template <int DA, int DB>
static hipError_t launch_mfma_one(const FpPrime* fprimes, const MacArgs& g, const int8_t* wd, int K, int K_pad, int OC_pad,
                                  const double* c3, dim3 grid, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    hipLaunchKernelGGL((scalar_mac_mfma_kernel<DA, DB>), grid, dim3(256), 0, st, fprimes, g, wd, K, K_pad, OC_pad, c3, log_n);
    return hipGetLastError();
}

// da: digits the weights need (1..7); db: digits the residues need (6: every prime below 2^46, else 7)
static hipError_t launch_scalar_mac_mfma(hisa_ctx* ctx, const FpPrime* fprimes, const MacArgs& g, const int8_t* wd, int K, int K_pad, int OC_pad,
                                         const double* c3, int da, int db, int batch, int log_n, hipStream_t st) {
    count_mac(g, batch, false);
    DRY_RUN_RETURN();
    if (hipError_t be = mac_bounds(ctx, g, batch, false)) return be;
    if (!fprimes || !wd || !c3 || !g.out || g.n_taps <= 0 || g.n_taps > MAX_TAPS || K != g.n_taps * g.IC || K_pad % MT_K ||
        K_pad < K || OC_pad % MT_OC || OC_pad < g.OC || log_n < 6 || da < 1 || da > MAC_DIGITS || (db != 6 && db != 7) ||
        !mac_shape_ok(g, log_n))
        return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / MT_E, mac_polys(g) * g.l, batch * (OC_pad / MT_OC));
    ProfScope prof__("scalar_mac_mfma_kernel", st);
    if (da < 3) da = 3;
#define MFMA_CASE(A_, B_) if (da == A_ && db == B_) return launch_mfma_one<A_, B_>(fprimes, g, wd, K, K_pad, OC_pad, c3, grid, log_n, st)
    MFMA_CASE(3, 6); MFMA_CASE(4, 6); MFMA_CASE(5, 6); MFMA_CASE(6, 6); MFMA_CASE(7, 6);
    MFMA_CASE(3, 7); MFMA_CASE(4, 7); MFMA_CASE(5, 7); MFMA_CASE(6, 7); MFMA_CASE(7, 7);
#undef MFMA_CASE
    return hipErrorInvalidValue;
}

// Plaintexts [cnt][l][N] of eight-byte residues -> the limb-major form [l][cnt] of rows of N residues: a packed row holds,
// for every 128 residues, their 128 low 32-bit words followed by their 128 high 16-bit words (768 bytes); an unpacked one
// is as it was (packed: bit 0 limb 0, bit 1 the rest).
// One launch converts the plaintexts first .. first + gridDim.z - 1.
__global__ __launch_bounds__(NT) void pack_plain_kernel(const u64* src, char* dst, int l, int packed, u64 cnt, u64 first, int log_n) {
    const u64 n = (u64)1 << log_n;
    const u64 j = (u64)blockIdx.x * NT + threadIdx.x;
    const int limb = blockIdx.y;
    const u64 b0 = (packed & 1) ? 6 : 8, b1 = (packed & 2) ? 6 : 8, c = first + blockIdx.z;
    const bool pk = packed >> (limb ? 1 : 0) & 1;
    const u64 v = src[(c * l + limb) * n + j];
    char* row = dst + (limb ? b0 + (u64)(limb - 1) * b1 : 0) * n * cnt + c * (pk ? 6 : 8) * n;
    if (pk) {
        *(uint32_t*)(row + (j >> 7) * 768 + (j & 127) * 4) = (uint32_t)v;
        *(uint16_t*)(row + (j >> 7) * 768 + 512 + (j & 127) * 2) = (uint16_t)(v >> 32);
    } else {
        ((u64*)row)[j] = v;
    }
}

static hipError_t launch_plain_mac_fp(hisa_ctx* ctx, const FpPrime* fprimes, const MacArgs& g, int batch, int log_n, hipStream_t st) {
    count_mac(g, batch, true);
    DRY_RUN_RETURN();
    if (hipError_t be = mac_bounds(ctx, g, batch, true)) return be;
    if (!fprimes || !g.w || !g.out || g.n_taps <= 0 || g.n_taps > MAX_TAPS || !mac_shape_ok(g, log_n)) return hipErrorInvalidValue;
    if (g.w_words && (u64)g.l * ((u64)1 << log_n) > g.w_words) return hipErrorInvalidValue;   // plaintexts shorter than the limbs walked
    if (g.x2 && (!g.out2 || g.lq <= 0 || g.lq > g.l || g.x2_words == 0)) return hipErrorInvalidValue;
    if (g.w_count) {   // limb-major plaintexts: of exactly the limbs walked, on the primes q_0.., no second input
        const u64 last = ((u64)g.n_taps * g.IC - 1) * g.w_stride_t + (u64)(g.OC - 1) * g.w_stride_oc;
        if (g.w_words || g.x2 || g.lq || g.polys == 1 || (g.w_packed & ~3) || last >= g.w_count || log_n < 9)
            return hipErrorInvalidValue;
    }
    const int ocp = (g.OC >= 8 && !g.w_count) ? 8 : 4;   // two coefficients per thread: four outputs fill the registers
    if ((u64)batch * ((g.OC + ocp - 1) / ocp) > 65535) return hipErrorInvalidValue;
    // the limb-major forms take two coefficients per thread
    dim3 grid((1u << log_n) / NT / (g.w_count ? 2 : 1), batch * ((g.OC + ocp - 1) / ocp), g.l);
    ProfScope prof__("plain_mac_fp_kernel", st);
    if (g.w_count) hipLaunchKernelGGL((plain_mac_fp_kernel<false, 4, true>), grid, dim3(NT), 0, st, fprimes, g, log_n);
    else if (g.x2 && ocp == 8) hipLaunchKernelGGL((plain_mac_fp_kernel<true, 8>), grid, dim3(NT), 0, st, fprimes, g, log_n);
    else if (g.x2) hipLaunchKernelGGL((plain_mac_fp_kernel<true, 4>), grid, dim3(NT), 0, st, fprimes, g, log_n);
    else if (ocp == 8) hipLaunchKernelGGL((plain_mac_fp_kernel<false, 8>), grid, dim3(NT), 0, st, fprimes, g, log_n);
    else hipLaunchKernelGGL((plain_mac_fp_kernel<false, 4>), grid, dim3(NT), 0, st, fprimes, g, log_n);
    return hipGetLastError();
}

static hipError_t launch_plain_mac(hisa_ctx* ctx, const PrimeConst* primes, const MacArgs& g, int batch, int log_n, hipStream_t st) {
    count_mac(g, batch, true);
    DRY_RUN_RETURN();
    if (hipError_t be = mac_bounds(ctx, g, batch, true)) return be;
    // the integer kernels know two-polynomial entries on the primes q_0.. only
    if (!primes || !g.w || !g.out || g.n_taps <= 0 || g.n_taps > MAX_TAPS || g.polys == 1 || g.lq || g.x2 || g.w_words ||
        !mac_shape_ok(g, log_n))
        return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / NT, g.l, batch * g.OC);
    ProfScope prof__("plain_mac_kernel", st);
    hipLaunchKernelGGL(plain_mac_kernel, grid, dim3(NT), 0, st, primes, g, log_n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------
// channels per ciphertext (0 in a zero-initialised struct means HW-tiling), ciphertexts per image, ciphertexts in all
static inline uint32_t t_ci(const hisa_tensor* t) { return t->c_inner ? t->c_inner : 1; }
static inline size_t t_per(const hisa_tensor* t) { return ((size_t)t->channels + t_ci(t) - 1) / t_ci(t); }
static inline size_t t_ncts(const hisa_tensor* t) { return (size_t)t->batch * t_per(t); }
// slot of the last element of a ciphertext
static inline u64 t_last(const hisa_tensor* t) {
    return (u64)t->offset + (u64)(t_ci(t) - 1) * t->c_stride + (u64)(t->height - 1) * t->h_stride +
           (u64)(t->width - 1) * t->w_stride;
}

static int check_layout(hisa_ctx* ctx, const hisa_tensor* t) {
    if (!t || !t->cts || t->batch == 0 || t->channels == 0 || t->height == 0 || t->width == 0)
        return fail(ctx, HISA_ERR_ARG, "empty tensor");
    if (t_ci(t) > 1 && t->c_stride == 0) return fail(ctx, HISA_ERR_ARG, "several channels per ciphertext need a channel stride");
    if (t_last(t) >= ctx->N / 2) return fail(ctx, HISA_ERR_ARG, "tensor elements do not fit the %u slots", ctx->N / 2);
    return HISA_OK;
}

static int check_tensor(hisa_ctx* ctx, const hisa_tensor* t) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_layout(ctx, t));
    return check_batch_shape(ctx, (const hisa_ct* const*)t->cts, t_ncts(t), 2);
}

// the layers that read neighbouring slots of one channel are written for one channel per ciphertext
static int require_hw_tiling(hisa_ctx* ctx, const hisa_tensor* t, const char* what) {
    if (t && t_ci(t) > 1) return fail(ctx, HISA_ERR_ARG, "%s takes HW-tiled tensors (one channel per ciphertext)", what);
    return HISA_OK;
}

static void free_handles(hisa_ctx* ctx, std::vector<hisa_ct*>& v) {
    for (hisa_ct* c : v) hisa_free(ctx, c);
    v.clear();
}

static int32_t norm_step(const hisa_ctx* ctx, i64 r) {
    const i64 slots = ctx->N / 2;
    r %= slots;
    if (r < 0) r += slots;
    return (int32_t)r;
}

// Rotation amounts of a convolution, one per (tap, d): HW-tiling has d = 0 only; with c_inner channel blocks per
// ciphertext the blocks are combined along diagonals (output block b reads input block (b + d) mod c_inner), so every
// tap is also rotated by d blocks.
// A CHW-tiled convolution may instead reduce over the channel blocks after the multiplication
// (HISA_CHW_ROTATE_SUMS): the inputs are then rotated by the taps only and the c_inner sums by d blocks.
static bool conv_rotates_sums(const hisa_tensor* in, const hisa_conv_geom* g) {
    return t_ci(in) > 1 && (g->chw_schedule == HISA_CHW_ROTATE_SUMS || g->chw_schedule == HISA_CHW_ROTATE_SUMS_TAPS);
}
// ... or the other way round (HISA_CHW_ROTATE_SUMS_TAPS): the inputs by the d blocks only, the per-tap sums by the taps
static bool conv_sums_by_taps(const hisa_tensor* in, const hisa_conv_geom* g) {
    return t_ci(in) > 1 && g->chw_schedule == HISA_CHW_ROTATE_SUMS_TAPS;
}

static int32_t conv_tap_amount(const hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, uint32_t fy, uint32_t fx) {
    const i64 ph = g->pad_same ? g->fh / 2 : 0, pw = g->pad_same ? g->fw / 2 : 0;
    return norm_step(ctx, ((i64)fy - ph) * in->h_stride + ((i64)fx - pw) * in->w_stride);
}

// rotations of the inputs
static std::vector<int32_t> conv_tap_steps(const hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g) {
    std::vector<int32_t> steps;
    if (conv_sums_by_taps(in, g)) {
        for (uint32_t d = 0; d < t_ci(in); d++) steps.push_back(norm_step(ctx, (i64)d * in->c_stride));
        return steps;
    }
    const uint32_t diagonals = conv_rotates_sums(in, g) ? 1 : t_ci(in);
    for (uint32_t fy = 0; fy < g->fh; fy++)
        for (uint32_t fx = 0; fx < g->fw; fx++)
            for (uint32_t d = 0; d < diagonals; d++)
                steps.push_back(norm_step(ctx, (i64)conv_tap_amount(ctx, in, g, fy, fx) + (i64)d * in->c_stride));
    return steps;
}

// Rotations of the sums when they are rotated: the diagonals 1 .. c_inner-1 (HISA_CHW_ROTATE_SUMS), or the filter taps
// in the order their sums are kept (HISA_CHW_ROTATE_SUMS_TAPS): the unrotated tap first, then the others row by row;
// sum_taps receives that order (filter tap index fy * fw + fx per sum).
static std::vector<int32_t> conv_sum_steps(const hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g,
                                           std::vector<uint32_t>* sum_taps = nullptr) {
    std::vector<int32_t> steps;
    if (conv_sums_by_taps(in, g)) {
        std::vector<uint32_t> order;
        for (int pass = 0; pass < 2; pass++)
            for (uint32_t fy = 0; fy < g->fh; fy++)
                for (uint32_t fx = 0; fx < g->fw; fx++) {
                    const int32_t a = conv_tap_amount(ctx, in, g, fy, fx);
                    if ((a == 0) == (pass == 0)) {
                        order.push_back(fy * g->fw + fx);
                        if (a) steps.push_back(a);
                    }
                }
        if (sum_taps) *sum_taps = order;
    } else if (conv_rotates_sums(in, g)) {
        for (uint32_t d = 1; d < t_ci(in); d++) steps.push_back(norm_step(ctx, (i64)d * in->c_stride));
    }
    return steps;
}

// The block rotation above wraps around cyclically only if the blocks fill the slot vector; otherwise a copy of the
// blocks is first placed behind them (rotRight by this amount and add).  0: not needed.  -1: no room for the copy.
static i64 conv_wrap_amount(const hisa_ctx* ctx, const hisa_tensor* in) {
    const u64 span = (u64)t_ci(in) * in->c_stride, slots = ctx->N / 2;
    if (t_ci(in) == 1 || span == slots) return 0;
    return 2 * span <= slots ? (i64)span : -1;
}

static int write_steps(const std::vector<int32_t>& all, int32_t* steps, size_t cap, size_t* n) {
    std::set<int32_t> uniq;
    for (int32_t s : all)
        if (s != 0) uniq.insert(s);
    if (!n) return HISA_ERR_ARG;
    *n = uniq.size();
    if (steps) {
        size_t i = 0;
        for (int32_t s : uniq) {
            if (i >= cap) return HISA_ERR_ARG;
            steps[i++] = s;
        }
    }
    return HISA_OK;
}

extern "C" int hisa_conv2d_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* geom, int32_t* steps,
                                     size_t cap, size_t* n) {
    if (!ctx || !in || !geom) return HISA_ERR_ARG;
    std::vector<int32_t> all = conv_tap_steps(ctx, in, geom);
    for (int32_t st : conv_sum_steps(ctx, in, geom)) all.push_back(st);
    const i64 wrap = conv_wrap_amount(ctx, in);
    if (wrap > 0) all.push_back(norm_step(ctx, -wrap));
    return write_steps(all, steps, cap, n);
}

// Rotation amounts of the rotate-and-add that brings the sum over a plane into slot `offset`.  Strided form:
// w_stride * 2^k then h_stride * 2^k, each dimension rounded up to a power of two (the extra positions are zero after
// the masked multiply); it needs padded rows that do not overlap and a padded plane that does not wrap around the
// slot vector.  Otherwise, or when it is not shorter: the contiguous window 1, 2, 4, .. covering the plane.
// With several channels per ciphertext the channel stride is a third strided dimension (c_stride * 2^k) under the
// same conditions; the padded elements have to stay below slot `limit`.
static std::vector<i64> reduce_steps(const hisa_tensor* in, u64 limit) {
    const uint32_t ci = t_ci(in);
    const u64 span = t_last(in) - in->offset;
    std::vector<i64> window;
    while (((u64)1 << window.size()) < span + 1) window.push_back((i64)1 << window.size());
    int wl = 0, hl = 0, cl = 0;
    while (((u64)1 << wl) < in->width) wl++;
    while (((u64)1 << hl) < in->height) hl++;
    while (((u64)1 << cl) < ci) cl++;
    const u64 last = (u64)in->offset + (((u64)1 << cl) - 1) * in->c_stride + (((u64)1 << hl) - 1) * in->h_stride +
                     (((u64)1 << wl) - 1) * in->w_stride;
    const bool fits = ((u64)in->w_stride << wl) <= in->h_stride && (ci == 1 || ((u64)in->h_stride << hl) <= in->c_stride) &&
                      last < limit;
    std::vector<i64> strided;
    for (int k = 0; k < wl; k++) strided.push_back((i64)in->w_stride << k);
    for (int k = 0; k < hl; k++) strided.push_back((i64)in->h_stride << k);
    for (int k = 0; k < cl; k++) strided.push_back((i64)in->c_stride << k);
    return (fits && strided.size() < window.size()) ? strided : window;
}

static std::vector<i64> fc_reduce_steps(const hisa_ctx* ctx, const hisa_tensor* in) { return reduce_steps(in, ctx->N / 2); }

// Steps s, 2s, 4s, .. of a rotate-and-add chain add up all multiples of s below 2^k s: up to ctx->merge_doublings
// consecutive doublings become one group of the 2^c - 1 amounts s, 2s, 3s, .. that is summed in one call
// (hisa_set_merge_doublings).  Every other step is a group of its own.
static std::vector<std::vector<i64>> merge_doublings(const hisa_ctx* ctx, const std::vector<i64>& steps) {
    std::vector<std::vector<i64>> groups;
    const size_t merge = ctx->merge_doublings;
    for (size_t i = 0; i < steps.size();) {
        size_t c = 1;
        while (merge >= 2 && c < merge && i + c < steps.size() && steps[i + c] == 2 * steps[i + c - 1]) c++;
        std::vector<i64> grp;
        if (c == 1) grp.push_back(steps[i]);
        else
            for (i64 m = 1; m < ((i64)1 << c); m++) grp.push_back(m * steps[i]);
        groups.push_back(grp);
        i += c;
    }
    return groups;
}

extern "C" int hisa_set_merge_doublings(hisa_ctx* ctx, uint32_t max_doublings) {
    if (!ctx) return HISA_ERR_ARG;
    if (max_doublings == 1 || max_doublings > 4) return fail(ctx, HISA_ERR_ARG, "max_doublings is 0 or 2..4");
    if (max_doublings && !fused_key_switch_available(ctx))
        return fail(ctx, HISA_ERR_ARG, "sums of rotations need the fused key-switch path (N >= 2^12, every prime below 2^50, dnum <= 8)");
    ctx->merge_doublings = max_doublings;
    return HISA_OK;
}

extern "C" int hisa_fc_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, int32_t* steps, size_t cap, size_t* n) {
    if (!ctx || !in) return HISA_ERR_ARG;
    std::vector<int32_t> all;
    for (const auto& grp : merge_doublings(ctx, fc_reduce_steps(ctx, in)))
        for (i64 r : grp) all.push_back(norm_step(ctx, r));
    return write_steps(all, steps, cap, n);
}

extern "C" int hisa_pool_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, int32_t* steps, size_t cap, size_t* n) {
    if (!ctx || !in) return HISA_ERR_ARG;
    std::vector<int32_t> all = {norm_step(ctx, in->w_stride), norm_step(ctx, in->h_stride),
                                norm_step(ctx, (i64)in->h_stride + in->w_stride)};
    return write_steps(all, steps, cap, n);
}

// slots of the elements of a plane
static std::vector<uint32_t> plane_slots(uint32_t h, uint32_t w, uint32_t hs, uint32_t ws, uint32_t off) {
    std::vector<uint32_t> s;
    for (uint32_t y = 0; y < h; y++)
        for (uint32_t x = 0; x < w; x++) s.push_back(off + y * hs + x * ws);
    return s;
}

// slots of the elements of one ciphertext, channel-major
static std::vector<uint32_t> tensor_slots(const hisa_tensor* t) {
    std::vector<uint32_t> s;
    for (uint32_t c = 0; c < t_ci(t); c++)
        for (uint32_t v : plane_slots(t->height, t->width, t->h_stride, t->w_stride, t->offset + c * t->c_stride)) s.push_back(v);
    return s;
}

// Encodes n_pts slot vectors that are non-zero only on `slots` (values[n_pts][slots.size()], host) into
// NTT-form plaintexts out[n_pts][limbs][N] (device).
static int encode_sparse_batch(hisa_ctx* ctx, const std::vector<uint32_t>& slots, const double* values, size_t n_pts,
                               double scale, int limbs, u64* out) {
    const size_t nnz = slots.size(), n = ctx->N;
    std::vector<uint32_t> g(nnz);
    const uint32_t mask = 2 * ctx->N - 1;
    for (size_t i = 0; i < nnz; i++) {
        uint32_t e = 1, b = 5, k = slots[i];
        for (; k; k >>= 1, b = (b * b) & mask)
            if (k & 1) e = (e * b) & mask;
        g[i] = e;
    }
    // Many non-zero slots (an image plane): the O(N log N) transform over the slot order, the values scattered into
    // dense rows on the device.  Few (a mask row, a weight on a handful of positions): the direct sum over them.
    const bool fft = nnz > 256;
    if (fft) g.assign(slots.begin(), slots.end());
    const size_t group = fft ? std::min<size_t>(n_pts, 256) : 0;   // plaintexts per transform launch (16 bytes per slot each)
    Temp dg(ctx, nnz * sizeof(uint32_t));
    Temp dv(ctx, n_pts * nnz * sizeof(double));
    Temp co(ctx, n_pts * n * sizeof(i64));
    Temp work(ctx, group * (n / 2) * 2 * sizeof(double), fft);
    if (!dg.ok() || !dv.ok() || !co.ok() || (fft && !work.ok())) return HISA_ERR_OOM;
    HIP_TRY(ctx, hipMemcpyAsync(dg.blk->ptr, g.data(), nnz * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(dv.blk->ptr, values, n_pts * nnz * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (fft) {
        for (size_t p0 = 0; p0 < n_pts; p0 += group) {
            const int cnt = (int)std::min<size_t>(group, n_pts - p0);
            HIP_TRY(ctx, launch_encode_fft(ctx->d_cos, ctx->d_sin, ctx->d_pow5, dv.as<double>() + p0 * nnz, nullptr, dg.as<uint32_t>(),
                                           (int)nnz, cnt, 2.0 * scale / (double)n, work.blk->ptr, co.as<i64>() + p0 * n,
                                           (int)ctx->log_n, ctx->stream));
            HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co.as<i64>() + p0 * n, out + p0 * limbs * n, limbs, cnt,
                                           (int)ctx->log_n, ctx->stream));
        }
    }
    // grid.y carries the plaintext index: stay below its limit
    for (size_t p0 = 0; !fft && p0 < n_pts; p0 += 32768) {
        const int cnt = (int)std::min<size_t>(32768, n_pts - p0);
        HIP_TRY(ctx, launch_encode(ctx->d_cos, ctx->d_sin, dg.as<uint32_t>(), dv.as<double>() + p0 * nnz, nullptr, (int)nnz,
                                   cnt, 2.0 * scale / (double)n, co.as<i64>() + p0 * n, (int)ctx->log_n, ctx->stream));
        HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co.as<i64>() + p0 * n, out + p0 * limbs * n, limbs, cnt,
                                       (int)ctx->log_n, ctx->stream));
    }
    for (size_t p0 = 0; p0 < n_pts; p0 += 4096)
        HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, out + p0 * limbs * n, (u64)limbs * n,
                                (int)(std::min<size_t>(4096, n_pts - p0) * limbs), identity_map(limbs), ctx->stream));
    return HISA_OK;
}

// Encodes n_pts slot vectors that are constant on each of nb slot sets (values[n_pts][nb], host; sets[b] = the slots
// of set b) and zero elsewhere into NTT-form plaintexts out[n_pts][limbs][N] (device): the same numbers as
// encode_sparse_batch up to the rounding order of the fp64 sums, at nb instead of (number of slots) terms per
// coefficient.
// Residues of n_pts signed coefficient vectors (device, [n_pts][N]) in NTT form: on q_0..q_{limbs-1}, and with `ext`
// also on the K special primes behind them (out[n_pts][limbs (+K)][N]: the limbs of a key-switch accumulator).
static int coeffs_to_ntt(hisa_ctx* ctx, const i64* co, size_t n_pts, int limbs, bool ext, u64* out) {
    const size_t n = ctx->N;
    const int K = ext ? (int)ctx->K : 0, tot = limbs + K;
    HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes, co, out, limbs, tot, (int)n_pts, (int)ctx->log_n, ctx->stream));
    if (ext)
        HIP_TRY(ctx, launch_reduce_i64(ctx->d_primes + ctx->L, co, out + (size_t)limbs * n, K, tot, (int)n_pts, (int)ctx->log_n,
                                       ctx->stream));
    PolyMap pm = identity_map(tot);
    for (int m = 0; m < K; m++) pm.prime_of[limbs + m] = (int16_t)(ctx->L + m);
    for (size_t q0 = 0; q0 < n_pts; q0 += 4096)
        HIP_TRY(ctx, launch_ntt(ctx->tabs, (int)ctx->log_n, out + q0 * tot * n, (u64)tot * n,
                                (int)(std::min<size_t>(4096, n_pts - q0) * tot), pm, ctx->stream));
    return HISA_OK;
}

static int encode_piecewise_batch(hisa_ctx* ctx, const std::vector<std::vector<uint32_t>>& sets, const double* values,
                                  size_t n_pts, double scale, int limbs, u64* out, bool ext = false) {
    const size_t n = ctx->N, nb = sets.size();
    std::vector<uint32_t> g;
    std::vector<int> begin(1, 0);
    const uint32_t mask = 2 * ctx->N - 1;
    for (const auto& set : sets) {
        for (uint32_t slot : set) {
            uint32_t e = 1, b = 5;
            for (uint32_t k = slot; k; k >>= 1, b = (b * b) & mask)
                if (k & 1) e = (e * b) & mask;
            g.push_back(e);
        }
        begin.push_back((int)g.size());
    }
    Temp dg(ctx, std::max<size_t>(1, g.size()) * sizeof(uint32_t)), db(ctx, begin.size() * sizeof(int));
    Temp basis(ctx, nb * n * sizeof(double)), dv(ctx, n_pts * nb * sizeof(double));
    if (!dg.ok() || !db.ok() || !basis.ok() || !dv.ok()) return HISA_ERR_OOM;
    HIP_TRY(ctx, hipMemcpyAsync(dg.blk->ptr, g.data(), g.size() * sizeof(uint32_t), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(db.blk->ptr, begin.data(), begin.size() * sizeof(int), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(dv.blk->ptr, values, n_pts * nb * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, launch_encode_basis(ctx->d_cos, dg.as<uint32_t>(), db.as<int>(), (int)nb, basis.as<double>(), (int)ctx->log_n,
                                     ctx->stream));
    const size_t chunk = std::min<size_t>(32768, std::max<size_t>(1, ((size_t)512 << 20) / (n * sizeof(i64))));
    Temp co(ctx, std::min(chunk, n_pts) * n * sizeof(i64));
    if (!co.ok()) return HISA_ERR_OOM;
    for (size_t p0 = 0; p0 < n_pts; p0 += chunk) {
        const size_t cnt = std::min(chunk, n_pts - p0);
        HIP_TRY(ctx, launch_encode_combine(basis.as<double>(), (int)nb, dv.as<double>() + p0 * nb, (int)cnt,
                                           2.0 * scale / (double)n, co.as<i64>(), (int)ctx->log_n, ctx->stream));
        TRY(coeffs_to_ntt(ctx, co.as<i64>(), cnt, limbs, ext, out + p0 * (limbs + (ext ? ctx->K : 0)) * n));
    }
    return HISA_OK;
}

// host signed coefficients [n_pts][N] -> NTT-form plaintexts out[n_pts][limbs][N]
static int coeffs_to_plain_batch(hisa_ctx* ctx, const int64_t* host, size_t n_pts, int limbs, u64* out, bool ext = false) {
    const size_t n = ctx->N, tot = limbs + (ext ? ctx->K : 0);
    for (size_t p0 = 0; p0 < n_pts; p0 += 4096) {
        const size_t cnt = std::min<size_t>(4096, n_pts - p0);
        Temp co(ctx, cnt * n * sizeof(i64));
        if (!co.ok()) return HISA_ERR_OOM;
        HIP_TRY(ctx, hipMemcpyAsync(co.blk->ptr, host + p0 * n, cnt * n * sizeof(i64), hipMemcpyHostToDevice, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        TRY(coeffs_to_ntt(ctx, co.as<i64>(), cnt, limbs, ext, out + p0 * tot * n));
    }
    return HISA_OK;
}

static u64 mod_i64(i64 v, u64 q) {
    if (v >= 0) return (u64)v % q;
    u64 m = ((u64)(-(v + 1)) + 1) % q;
    return m ? q - m : 0;
}

static void fill_out_meta(hisa_tensor* out, uint32_t batch, uint32_t channels, uint32_t h, uint32_t w, uint32_t hs,
                          uint32_t ws, uint32_t off, uint32_t clean, uint32_t c_inner = 1, uint32_t c_stride = 0) {
    out->batch = batch; out->channels = channels; out->height = h; out->width = w;
    out->h_stride = hs; out->w_stride = ws; out->offset = off; out->clean = clean;
    out->c_inner = c_inner; out->c_stride = c_stride;
}

// ---------------------------------------------------------------------------
// conv2d
// ---------------------------------------------------------------------------
struct ConvPlan {
    uint32_t out_h, out_w;
    std::vector<int32_t> steps;   // rotations of the inputs: one per (tap, d), or per tap when the sums are rotated
    std::vector<int32_t> sum_steps;   // the rotations of the sums, where sums are rotated (conv_sum_steps)
    std::vector<uint32_t> sum_taps;   // HISA_CHW_ROTATE_SUMS_TAPS: filter tap of every sum, the unrotated ones first
    bool rotate_sums = false, sums_by_taps = false;
    i64 wrap = 0;                 // CHW-tiling: rotRight amount of the copy behind the channel blocks, 0 if none
};

static int conv_plan(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, ConvPlan* p) {
    if (!g || g->chw_schedule > HISA_CHW_ROTATE_SUMS_TAPS) return fail(ctx, HISA_ERR_ARG, "bad conv geometry");
    p->rotate_sums = conv_rotates_sums(in, g);
    p->sums_by_taps = conv_sums_by_taps(in, g);
    const u64 input_rotations = p->sums_by_taps ? t_ci(in) : (u64)g->fh * g->fw * (p->rotate_sums ? 1 : t_ci(in));
    if (g->fh == 0 || g->fw == 0 || g->stride == 0 || input_rotations > MAX_TAPS || g->mode > HISA_CONV_PLAIN)
        return fail(ctx, HISA_ERR_ARG, "bad conv geometry (at most %d rotation amounts per input ciphertext)", MAX_TAPS);
    if (p->rotate_sums) {
        if (!fused_key_switch_available(ctx))
            return fail(ctx, HISA_ERR_ARG, "rotating the sums needs the fused key-switch path (N >= 2^12, every prime below 2^50, dnum <= 8)");
        if ((p->sums_by_taps ? (u64)g->fh * g->fw : (u64)t_ci(in)) - 1 > FP_MAX_STEPS)
            return fail(ctx, HISA_ERR_ARG, "rotating the sums: at most %d sums per output ciphertext", FP_MAX_STEPS + 1);
        if (g->shared_moddown) return fail(ctx, HISA_ERR_ARG, "shared_moddown belongs to the schedule that rotates the inputs");
    }
    if (t_ci(in) > 1) {
        // several channels per ciphertext: different weights on different slots, so mulPlain, and zeros between the elements
        if (g->mode != HISA_CONV_PLAIN) return fail(ctx, HISA_ERR_ARG, "CHW-tiled convolution multiplies by plaintexts: mode HISA_CONV_PLAIN");
        if (!in->clean) return fail(ctx, HISA_ERR_ARG, "CHW-tiled convolution needs a clean input tensor (hisa_tensor_mask makes one)");
        p->wrap = conv_wrap_amount(ctx, in);
        if (p->wrap < 0) return fail(ctx, HISA_ERR_ARG, "the channel blocks must fill the slots or leave room for one copy behind them");
    }
    if (g->pad_same > HISA_PAD_SAME_MASKED) return fail(ctx, HISA_ERR_ARG, "bad padding");
    if (g->pad_same == HISA_PAD_SAME_MASKED && (g->mode != HISA_CONV_PLAIN || g->shared_moddown || t_ci(in) == 1))
        return fail(ctx, HISA_ERR_ARG, "SAME padding by masking is for CHW-tiled tensors (HISA_CONV_PLAIN, no shared_moddown)");
    if (g->pad_same) {
        if (g->pad_same == HISA_PAD_SAME && !in->clean)
            return fail(ctx, HISA_ERR_ARG, "SAME padding needs a clean input tensor (zeros around the plane)");
        p->out_h = (in->height + g->stride - 1) / g->stride;
        p->out_w = (in->width + g->stride - 1) / g->stride;
    } else {
        if (in->height < g->fh || in->width < g->fw) return fail(ctx, HISA_ERR_ARG, "filter larger than the plane");
        p->out_h = (in->height - g->fh) / g->stride + 1;
        p->out_w = (in->width - g->fw) / g->stride + 1;
    }
    p->steps = conv_tap_steps(ctx, in, g);
    p->sum_steps = conv_sum_steps(ctx, in, g, &p->sum_taps);
    if (p->sums_by_taps && p->sum_steps.size() + 1 != (size_t)g->fh * g->fw)
        return fail(ctx, HISA_ERR_ARG, "rotating the sums by the taps needs exactly one tap without a rotation");
    return HISA_OK;
}

// Fixed-point weights w[K][OC] (K = taps x input channels) on the device: residues per limb for the integer kernel;
// when every prime is below 2^50 also centred doubles [l][K][OC] for the fp64 kernel and, for contractions long enough
// to fill the matrix cores, signed base-256 digits [l][7][OC_pad][K_pad] with the constants 2^(24 g) mod q.
#define MFMA_MIN_K 32
#define MFMA_MAX_K 16384   // 7 K 2^14 must stay below 2^31
struct DevWeights {
    size_t K, OC, K_pad, OC_pad;
    int da = MAC_DIGITS;   // signed base-256 digits the largest weight needs
    bool fp, mfma;
    std::vector<int> primes;   // prime of every limb position (empty: position i is prime i)
    Temp res, resf, digits, c3;
    DevWeights(hisa_ctx* ctx, size_t K_, size_t OC_, uint32_t l)
        : K(K_), OC(OC_), K_pad((K_ + MT_K - 1) / MT_K * MT_K), OC_pad((OC_ + MT_OC - 1) / MT_OC * MT_OC),
          fp(ctx->tabs.fp_ok), mfma(ctx->tabs.fp_ok && K_ >= MFMA_MIN_K && K_ <= MFMA_MAX_K),
          res(ctx, K_ * OC_ * l * sizeof(u64)), resf(ctx, fp ? K_ * OC_ * l * sizeof(double) : 8),
          digits(ctx, mfma ? (size_t)l * MAC_DIGITS * OC_pad * K_pad : 8), c3(ctx, mfma ? (size_t)l * 5 * sizeof(double) : 8) {}
    bool ok() const { return res.ok() && resf.ok() && digits.ok() && c3.ok(); }
};

static int upload_weight_residues(hisa_ctx* ctx, const int64_t* w_int, uint32_t l, DevWeights& dst) {
    const size_t count = dst.K * dst.OC;
    std::vector<u64> res(count * l);
    std::vector<double> resf(dst.fp ? count * l : 0), c3(dst.mfma ? (size_t)l * 5 : 0);
    std::vector<int8_t> dig(dst.mfma ? (size_t)l * MAC_DIGITS * dst.OC_pad * dst.K_pad : 0, 0);
    u64 used = 0;   // OR of all digit words: its highest non-zero byte is the last digit in use
    for (uint32_t k = 0; k < l; k++) {
        const u64 q = ctx->mod[dst.primes.empty() ? k : (uint32_t)dst.primes[k]];
        for (size_t oc = 0; oc < dst.OC; oc++) {       // digit rows are contiguous in the contraction index
            for (size_t kk = 0; kk < dst.K; kk++) {
                const size_t i = kk * dst.OC + oc;
                const i64 wv = w_int[i];
                // weights are almost always far below the modulus: the remainder is then the value itself
                const u64 r = (wv >= 0 && (u64)wv < q) ? (u64)wv : ((wv < 0 && wv > -(i64)q) ? q - (u64)(-wv) : mod_i64(wv, q));
                res[i * l + k] = r;
                if (!dst.fp) continue;
                const i64 c = r > q / 2 ? -(i64)(q - r) : (i64)r;
                resf[(size_t)k * count + i] = (double)c;   // [l][K][OC]
                if (!dst.mfma) continue;
                const u64 d = balanced_digits((u64)c);
                used |= d;
                int8_t* row = dig.data() + ((size_t)k * MAC_DIGITS * dst.OC_pad + oc) * dst.K_pad + kk;
                for (int a = 0; a < MAC_DIGITS; a++) row[(size_t)a * dst.OC_pad * dst.K_pad] = (int8_t)(uint8_t)(d >> (8 * a));
            }
        }
        if (dst.mfma) {
            u64 pw = 1 % q;
            for (int gq = 0; gq < 5; gq++) {
                c3[(size_t)k * 5 + gq] = pw > q / 2 ? -(double)(q - pw) : (double)pw;
                for (int i = 0; i < 24; i++) pw = (pw << 1) % q;
            }
        }
    }
    dst.da = 1;
    for (int a = 1; a < MAC_DIGITS; a++)
        if ((used >> (8 * a)) & 0xFF) dst.da = a + 1;
    HIP_TRY(ctx, hipMemcpyAsync(dst.res.blk->ptr, res.data(), res.size() * sizeof(u64), hipMemcpyHostToDevice, ctx->stream));
    if (dst.fp)
        HIP_TRY(ctx, hipMemcpyAsync(dst.resf.blk->ptr, resf.data(), resf.size() * sizeof(double), hipMemcpyHostToDevice,
                                    ctx->stream));
    if (dst.mfma) {
        HIP_TRY(ctx, hipMemcpyAsync(dst.digits.blk->ptr, dig.data(), dig.size(), hipMemcpyHostToDevice, ctx->stream));
        HIP_TRY(ctx, hipMemcpyAsync(dst.c3.blk->ptr, c3.data(), c3.size() * sizeof(double), hipMemcpyHostToDevice, ctx->stream));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return HISA_OK;
}

// The inputs of a convolution as its multiply-accumulate reads them: the gathered batch (with the copy of the channel
// blocks behind them where the layout needs it) and its rotations by the distinct non-zero amounts of `steps`, all from
// one hoisted call (one decomposition of c1).  Convolutions of the same tensor that ask for the same amounts can share
// one set (hisa_conv2d_apply_multi): a rotation computed once or twice has the same bits.
struct RotatedInputs {
    int32_t wrap = 0;
    std::vector<hisa_ct*> wrapped;
    BatchIn bi = {};
    std::vector<int32_t> steps;                    // distinct, non-zero
    std::vector<std::vector<hisa_ct*>> rotated;    // per entry of steps: the nct rotated ciphertexts (one allocation)
    const u64* base_of(int32_t step) const {
        if (step == 0) return bi.base;
        for (size_t k = 0; k < steps.size(); k++)
            if (steps[k] == step) return rotated[k].empty() ? nullptr : rotated[k][0]->data;
        return nullptr;
    }
};

static void release_inputs(hisa_ctx* ctx, RotatedInputs& r) {
    for (auto& v : r.rotated) free_handles(ctx, v);
    r.rotated.clear();
    r.steps.clear();
    dev_release(ctx, r.bi.tmp);
    r.bi = {};
    free_handles(ctx, r.wrapped);
    r.wrapped.clear();
}

static int rotate_inputs(hisa_ctx* ctx, const hisa_tensor* in, int32_t wrap, const std::vector<int32_t>& steps, RotatedInputs& r) {
    const uint32_t l = in->cts[0]->limbs;
    const size_t nct = (size_t)in->batch * t_per(in);
    r.wrap = wrap;
    hisa_ct* const* src = in->cts;
    if (wrap > 0) {
        r.wrapped.assign(nct, nullptr);
        TRY(hisa_rot_left_batch(ctx, (const hisa_ct* const*)in->cts, nct, norm_step(ctx, -wrap), r.wrapped.data()));
        BatchIn orig;
        int rcw = gather_batch(ctx, (const hisa_ct* const*)in->cts, nct, &orig);
        if (rcw == HISA_OK) {
            const u64 words = ct_words(ctx, 2, l);
            hipError_t e = launch_addsub(ctx->d_primes, r.wrapped[0]->data, orig.base, r.wrapped[0]->data, OP_ADD, (int)l, 2, 2, nct,
                                         words, orig.stride, words, (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rcw = fail(ctx, HISA_ERR_HIP, "conv wrap: %s", hipGetErrorString(e));
        }
        dev_release(ctx, orig.tmp);
        if (rcw != HISA_OK) { release_inputs(ctx, r); return rcw; }
        src = r.wrapped.data();
    }
    {
        const int rcg = gather_batch(ctx, (const hisa_ct* const*)src, nct, &r.bi);
        if (rcg != HISA_OK) { release_inputs(ctx, r); return rcg; }
    }
    for (int32_t st : steps)
        if (st != 0 && std::find(r.steps.begin(), r.steps.end(), st) == r.steps.end()) r.steps.push_back(st);
    if (!r.steps.empty()) {   // one call, so that the decomposition of c1 is shared by all amounts
        std::vector<hisa_ct*> all(r.steps.size() * nct, nullptr);
        const int rc = hisa_rot_left_hoisted_batch(ctx, (const hisa_ct* const*)src, nct, r.steps.data(), r.steps.size(), all.data());
        if (rc != HISA_OK) { release_inputs(ctx, r); return rc; }
        r.rotated.resize(r.steps.size());
        for (size_t k = 0; k < r.steps.size(); k++) r.rotated[k].assign(all.begin() + k * nct, all.begin() + (k + 1) * nct);
    }
    return HISA_OK;
}

// the rotated inputs of a plan's taps, from a shared set or made here
static int tap_inputs(hisa_ctx* ctx, const hisa_tensor* in, const ConvPlan& plan, const RotatedInputs* shared, RotatedInputs& own,
                      MacArgs& ma) {
    const RotatedInputs* ri = shared;
    if (!ri) {
        TRY(rotate_inputs(ctx, in, plan.wrap, plan.steps, own));
        ri = &own;
    } else if (ri->wrap != plan.wrap) {
        return fail(ctx, HISA_ERR_ARG, "shared rotations of another layout");
    }
    if (plan.steps.size() > MAX_TAPS) return fail(ctx, HISA_ERR_ARG, "too many taps");
    for (size_t t = 0; t < plan.steps.size(); t++) {
        ma.tap_base[t] = ri->base_of(plan.steps[t]);
        if (!ma.tap_base[t]) {
            if (!shared) release_inputs(ctx, own);
            return fail(ctx, HISA_ERR_ARG, "a rotation of the inputs is missing");
        }
    }
    return HISA_OK;
}

// dw: SCALAR/MASKED weights (null for PLAIN); d_pts: MASKED [l][N], PLAIN [T][OC][l][N]
static int conv_run(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, const ConvPlan& plan, uint32_t OC,
                    DevWeights* dw, double w_scale, const u64* d_pts, double pt_scale, hisa_tensor* out, u64 pt_count = 0,
                    int pt_packed = 0, const RotatedInputs* shared = nullptr) {
    // in units of ciphertexts: IC inputs and OCm outputs per image (HW-tiling: the channels themselves)
    const uint32_t B = in->batch, ci = t_ci(in), IC = (uint32_t)t_per(in), OCm = (OC + ci - 1) / ci, l = in->cts[0]->limbs;
    const size_t n = ctx->N;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "conv needs a level to rescale into");
    const int n_taps = (int)plan.steps.size();
    std::vector<hisa_ct*> outs((size_t)B * OCm, nullptr);
    MacArgs ma = {};
    RotatedInputs own;
    TRY(tap_inputs(ctx, in, plan, shared, own, ma));
    int rc = HISA_OK;
    const double in_scale = in->cts[0]->scale;
    double mac_scale = in_scale * (g->mode == HISA_CONV_PLAIN ? pt_scale : w_scale);
    if (rc == HISA_OK) rc = alloc_ct_batch(ctx, (size_t)B * OCm, 2, l, mac_scale, outs.data());
    if (rc == HISA_OK) {
        ma.n_taps = n_taps; ma.IC = (int)IC; ma.OC = (int)OCm; ma.l = (int)l; ma.ct_words = 2 * (u64)l * n;
        ma.out = outs[0]->data;
        hipError_t e;
        if (g->mode == HISA_CONV_PLAIN) {
            ma.w = d_pts; ma.w_stride_t = OCm; ma.w_stride_oc = 1; ma.w_count = pt_count; ma.w_packed = pt_packed;
            if (ctx->tabs.fp_ok) e = launch_plain_mac_fp(ctx, ctx->tabs.fprimes, ma, (int)B, (int)ctx->log_n, ctx->stream);
            else e = launch_plain_mac(ctx, ctx->d_primes, ma, (int)B, (int)ctx->log_n, ctx->stream);
        } else {
            ma.w = dw->res.u();
            if (dw->mfma) {
                u64 qmax = 0;
                for (uint32_t k = 0; k < l; k++) qmax = std::max(qmax, ctx->mod[k]);
                const int db = qmax < ((u64)1 << 46) ? 6 : 7;   // six balanced digits reach 0.498 * 2^48 (just under 2^47)
                e = launch_scalar_mac_mfma(ctx, ctx->tabs.fprimes, ma, (const int8_t*)dw->digits.blk->ptr, (int)dw->K, (int)dw->K_pad,
                                           (int)dw->OC_pad, dw->c3.as<double>(), dw->da, db, (int)B, (int)ctx->log_n, ctx->stream);
            }
            else if (dw->fp)
                e = launch_scalar_mac_fp(ctx, ctx->tabs.fprimes, ma, dw->resf.as<double>(), (int)B, (int)ctx->log_n, ctx->stream);
            else e = launch_scalar_mac(ctx, ctx->d_primes, ma, (int)B, (int)ctx->log_n, ctx->stream);
            if (e == hipSuccess && g->mode == HISA_CONV_MASKED) {
                e = launch_mul_plain(ctx->d_primes, outs[0]->data, d_pts, outs[0]->data, (int)l, 2, (u64)B * OC, ma.ct_words,
                                     ma.ct_words, (int)ctx->log_n, ctx->stream);
                for (hisa_ct* c : outs) c->scale = mac_scale * pt_scale;
            }
        }
        if (e != hipSuccess) rc = mac_fail(ctx, e, "conv");
    }
    if (!shared) release_inputs(ctx, own);
    if (rc == HISA_OK) rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    if (rc != HISA_OK) {
        for (hisa_ct* c : outs) hisa_free(ctx, c);
        return rc;
    }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    // unmasked outputs carry neighbour sums outside the valid positions, except for a 1x1 stride-1 filter
    const bool keeps_zeros = g->fh == 1 && g->fw == 1 && g->stride == 1 && in->clean;
    fill_out_meta(out, B, OC, plan.out_h, plan.out_w, in->h_stride * g->stride, in->w_stride * g->stride, in->offset,
                  (g->mode != HISA_CONV_SCALAR || keeps_zeros) ? 1u : 0u, ci, in->c_stride);
    return HISA_OK;
}

// CHW-tiled convolution that reduces over the channel blocks after the multiplication (HISA_CHW_ROTATE_SUMS):
// the inputs are rotated by the taps (one shared decomposition), one multiply-accumulate launch forms, for every
// output ciphertext g and diagonal d, the sum over (tap, input ciphertext) on the blocks where the input channels lie
// -- c_inner * OCm sums, ordered (d, g) -- and the sums of d = 1 .. c_inner-1 are rotated left by d blocks and added
// to the sum of d = 0 with one division by P per output (rotate_sum_fp).  d_pts: [taps][IC][c_inner * OCm][l][N].
// HISA_CHW_ROTATE_SUMS_TAPS exchanges the roles: the inputs are rotated by the d blocks, the sums (one per filter tap,
// the unrotated tap first) by the taps; d_pts: [c_inner][IC][taps * OCm][l][N].
static int conv_run_sums(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, const ConvPlan& plan, uint32_t OC,
                         const u64* d_pts, double pt_scale, hisa_tensor* out, u64 pt_count = 0, int pt_packed = 0,
                         const RotatedInputs* shared = nullptr) {
    const uint32_t B = in->batch, ci = t_ci(in), IC = (uint32_t)t_per(in), OCm = (OC + ci - 1) / ci, l = in->cts[0]->limbs;
    const size_t n = ctx->N;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "conv needs a level to rescale into");
    if (!d_pts || plan.sum_steps.size() != (plan.sums_by_taps ? plan.sum_taps.size() : (size_t)ci) - 1)
        return fail(ctx, HISA_ERR_ARG, "bad convolution plan");
    const int n_taps = (int)plan.steps.size();
    const u64 ctw = 2 * (u64)l * n;
    std::vector<hisa_ct*> outs((size_t)B * OCm, nullptr);
    MacArgs ma = {};
    RotatedInputs own;
    TRY(tap_inputs(ctx, in, plan, shared, own, ma));
    int rc = HISA_OK;
    const double mac_scale = in->cts[0]->scale * pt_scale;
    const size_t terms = plan.sum_steps.size() + 1;
    const size_t sums = terms * OCm;               // per image, ordered (term, g): term = diagonal d, or sum k of the taps
    Temp y(ctx, (size_t)B * sums * ctw * sizeof(u64));
    if (rc == HISA_OK && !y.ok()) rc = HISA_ERR_OOM;
    // with hisa_set_fused_rescale the sums come back divided by q_{l-1} P: one limb fewer, no divScalar afterwards
    const bool fused = ctx->fused_rescale != 0;
    if (rc == HISA_OK)
        rc = alloc_ct_batch(ctx, (size_t)B * OCm, 2, fused ? l - 1 : l, fused ? mac_scale / (double)ctx->mod[l - 1] : mac_scale,
                            outs.data());
    if (rc == HISA_OK) {
        ma.n_taps = n_taps; ma.IC = (int)IC; ma.OC = (int)sums; ma.l = (int)l; ma.ct_words = ctw;
        ma.out = y.u();
        ma.w = d_pts; ma.w_stride_t = sums; ma.w_stride_oc = 1; ma.w_count = pt_count; ma.w_packed = pt_packed;
        hipError_t e = launch_plain_mac_fp(ctx, ctx->tabs.fprimes, ma, (int)B, (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = mac_fail(ctx, e, "conv");
    }
    if (!shared) release_inputs(ctx, own);
    // per image: entries (d, g) are rotation-major over the OCm outputs; d = 0 is the unrotated term
    for (uint32_t b = 0; b < B && rc == HISA_OK; b++) {
        const u64* yb = y.u() + (size_t)b * sums * ctw;
        rc = rotate_sum_fp(ctx, yb + (size_t)OCm * ctw, ctw, (int)terms - 1, plan.sum_steps.data(), OCm, (int)l, yb, ctw,
                           outs[(size_t)b * OCm]->data, false, fused);
    }
    if (rc == HISA_OK && !fused) rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    if (rc != HISA_OK) {
        for (hisa_ct* c : outs) hisa_free(ctx, c);
        return rc;
    }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    fill_out_meta(out, B, OC, plan.out_h, plan.out_w, in->h_stride * g->stride, in->w_stride * g->stride, in->offset, 1u, ci,
                  in->c_stride);
    return HISA_OK;
}

// Everything a convolution needs besides its input: weights in the forms the kernels read, the mask or the per-tap
// plaintexts, and the scales.  Built from float weights per call by hisa_conv2d, or once by hisa_conv2d_prepare.
// With `shared` (one division by P per output ciphertext, conv_run_shared) the terms of the rotated taps and of the
// unrotated ones are kept apart, the former on the l + K limbs of the key-switch accumulators: dw / pts hold the
// rotated taps' weights ([T_rot][OC], plaintexts with l + K limbs), dw_zero / pts_zero the others (l limbs); the mask
// of MASKED mode is then in `mask`.
struct ConvWeights {
    DevWeights* dw = nullptr;   // SCALAR / MASKED
    Temp* pts = nullptr;        // MASKED: the mask [l][N]; PLAIN: [T][OC][l][N]
    double w_scale = 1.0, pt_scale = 1.0;
    bool shared = false;
    DevWeights* dw_zero = nullptr;
    Temp* pts_zero = nullptr;
    Temp* mask = nullptr;
    u64 pt_count = 0;           // PLAIN, converted by pack_plain_weights: plaintexts in the limb-major form (0: as encoded)
    int pt_packed = 0;          // which limbs have six-byte residues (MacArgs::w_packed)
    ~ConvWeights() { delete dw; delete pts; delete dw_zero; delete pts_zero; delete mask; }
};

// taps (entries of plan.steps) with and without a rotation
struct TapSplit { std::vector<int> rot, zero; };
static TapSplit split_taps(const ConvPlan& plan) {
    TapSplit t;
    for (size_t k = 0; k < plan.steps.size(); k++) (plan.steps[k] ? t.rot : t.zero).push_back((int)k);
    return t;
}

// rows (tap * rows_per_tap + r) of a [taps][rows_per_tap][items] array, for the listed taps
template <class T>
static std::vector<T> pick_taps(const T* src, const std::vector<int>& taps, size_t rows_per_tap, size_t items) {
    std::vector<T> out(taps.size() * rows_per_tap * items);
    for (size_t k = 0; k < taps.size(); k++)
        memcpy(out.data() + k * rows_per_tap * items, src + (size_t)taps[k] * rows_per_tap * items, rows_per_tap * items * sizeof(T));
    return out;
}

// Does this convolution take the shared-ModDown schedule?  Asked for and impossible is an error.
static int conv_wants_shared(hisa_ctx* ctx, const hisa_conv_geom* g, const ConvPlan& plan, bool* shared) {
    *shared = false;
    if (!g->shared_moddown) return HISA_OK;
    if (!fused_key_switch_available(ctx))
        return fail(ctx, HISA_ERR_ARG, "shared_moddown needs the fused key-switch path (N >= 2^12, every prime below 2^50, dnum <= 8)");
    if (t_analysis) return HISA_OK;      // dry runs count the term-by-term schedule
    for (int32_t st : plan.steps)
        if (st) *shared = true;
    return HISA_OK;
}

static std::vector<int> ext_prime_list(const hisa_ctx* ctx, uint32_t l) {
    std::vector<int> p;
    for (uint32_t i = 0; i < l; i++) p.push_back((int)i);
    for (uint32_t m = 0; m < ctx->K; m++) p.push_back((int)(ctx->L + m));
    return p;
}

// scalar weights w_int[T][OC] -> device forms; shared: split by tap, the rotated ones on the l + K limbs
static int build_scalar_weights(hisa_ctx* ctx, const int64_t* w_int, const ConvPlan& plan, uint32_t ICm, uint32_t OC, uint32_t l,
                                bool shared, ConvWeights& cw) {
    cw.shared = shared;
    if (!shared) {
        cw.dw = new DevWeights(ctx, plan.steps.size() * ICm, OC, l);
        if (!cw.dw->ok()) return HISA_ERR_OOM;
        return upload_weight_residues(ctx, w_int, l, *cw.dw);
    }
    const TapSplit ts = split_taps(plan);
    const std::vector<int64_t> wr = pick_taps(w_int, ts.rot, ICm, OC), wz = pick_taps(w_int, ts.zero, ICm, OC);
    cw.dw = new DevWeights(ctx, ts.rot.size() * ICm, OC, l + ctx->K);
    if (!cw.dw->ok()) return HISA_ERR_OOM;
    cw.dw->primes = ext_prime_list(ctx, l);
    TRY(upload_weight_residues(ctx, wr.data(), l + ctx->K, *cw.dw));
    if (!ts.zero.empty()) {
        cw.dw_zero = new DevWeights(ctx, ts.zero.size() * ICm, OC, l);
        if (!cw.dw_zero->ok()) return HISA_ERR_OOM;
        TRY(upload_weight_residues(ctx, wz.data(), l, *cw.dw_zero));
    }
    return HISA_OK;
}

// piecewise-constant plaintext weights vals[T][OCm][sets.size()] -> NTT-form plaintexts; shared: split as above
// per_tap (SAME padding by masking): the slot sets differ from filter tap to filter tap -- per_tap[tap] replaces `sets`
// for the plaintexts of that tap, which are contiguous (the tap is the outermost index of the plaintext order)
static int build_plain_weights(hisa_ctx* ctx, const std::vector<std::vector<uint32_t>>& sets, const double* vals,
                               const ConvPlan& plan, uint32_t ICm, uint32_t OCm, uint32_t l, double scale, bool shared,
                               ConvWeights& cw, const std::vector<std::vector<std::vector<uint32_t>>>* per_tap = nullptr) {
    const size_t n = ctx->N, nb = sets.size(), T = plan.steps.size() * ICm;
    cw.shared = shared;
    cw.pt_scale = scale;
    if (per_tap) {
        if (shared || per_tap->empty() || (T * OCm) % per_tap->size()) return fail(ctx, HISA_ERR_ARG, "bad plaintext layout");
        cw.pts = new Temp(ctx, T * OCm * l * n * sizeof(u64));
        if (!cw.pts->ok()) return HISA_ERR_OOM;
        const size_t rows = T * OCm / per_tap->size();
        for (size_t tap = 0; tap < per_tap->size(); tap++) {
            if ((*per_tap)[tap].size() != nb) return fail(ctx, HISA_ERR_ARG, "bad plaintext layout");
            TRY(encode_piecewise_batch(ctx, (*per_tap)[tap], vals + tap * rows * nb, rows, scale, (int)l,
                                       cw.pts->u() + tap * rows * l * n));
        }
        return HISA_OK;
    }
    if (!shared) {
        cw.pts = new Temp(ctx, T * OCm * l * n * sizeof(u64));
        if (!cw.pts->ok()) return HISA_ERR_OOM;
        return encode_piecewise_batch(ctx, sets, vals, T * OCm, scale, (int)l, cw.pts->u());
    }
    const TapSplit ts = split_taps(plan);
    const std::vector<double> vr = pick_taps(vals, ts.rot, ICm, OCm * nb), vz = pick_taps(vals, ts.zero, ICm, OCm * nb);
    cw.pts = new Temp(ctx, ts.rot.size() * ICm * OCm * (l + ctx->K) * n * sizeof(u64));
    if (!cw.pts->ok()) return HISA_ERR_OOM;
    TRY(encode_piecewise_batch(ctx, sets, vr.data(), ts.rot.size() * ICm * OCm, scale, (int)l, cw.pts->u(), true));
    if (!ts.zero.empty()) {
        cw.pts_zero = new Temp(ctx, ts.zero.size() * ICm * OCm * l * n * sizeof(u64));
        if (!cw.pts_zero->ok()) return HISA_ERR_OOM;
        TRY(encode_piecewise_batch(ctx, sets, vz.data(), ts.zero.size() * ICm * OCm, scale, (int)l, cw.pts_zero->u()));
    }
    return HISA_OK;
}

static int conv_build(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t OC, const hisa_conv_geom* geom,
                      const ConvPlan& plan, ConvWeights& cw) {
    const uint32_t l = in->cts[0]->limbs, IC = in->channels;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "conv needs a level to rescale into");
    const size_t taps = plan.steps.size(), T = taps * IC, n = ctx->N;
    const double q_last = (double)ctx->mod[l - 1];
    bool shared;
    TRY(conv_wants_shared(ctx, geom, plan, &shared));
    const std::vector<uint32_t> vslots = plane_slots(plan.out_h, plan.out_w, in->h_stride * geom->stride,
                                                     in->w_stride * geom->stride, in->offset);
    // SAME padding by masking: per filter tap, the outputs whose input element under that tap lies inside the plane
    const bool masked_same = geom->pad_same == HISA_PAD_SAME_MASKED;
    std::vector<std::vector<uint32_t>> tap_slots;
    if (masked_same) {
        for (uint32_t fy = 0; fy < geom->fh; fy++)
            for (uint32_t fx = 0; fx < geom->fw; fx++) {
                std::vector<uint32_t> here;
                for (uint32_t oy = 0; oy < plan.out_h; oy++)
                    for (uint32_t ox = 0; ox < plan.out_w; ox++) {
                        const i64 iy = (i64)oy * geom->stride + fy - geom->fh / 2, ix = (i64)ox * geom->stride + fx - geom->fw / 2;
                        if (iy >= 0 && iy < (i64)in->height && ix >= 0 && ix < (i64)in->width) here.push_back(vslots[(size_t)oy * plan.out_w + ox]);
                    }
                tap_slots.push_back(here);
            }
    }
    // the slot sets of the blocks at positions 0 .. npos-1 for every filter tap
    auto block_sets = [&](uint32_t npos) {
        std::vector<std::vector<std::vector<uint32_t>>> per_tap(tap_slots.size(), std::vector<std::vector<uint32_t>>(npos));
        for (size_t tap = 0; tap < tap_slots.size(); tap++)
            for (uint32_t pos = 0; pos < npos; pos++)
                for (uint32_t v : tap_slots[tap]) per_tap[tap][pos].push_back(v + pos * in->c_stride);
        return per_tap;
    };
    if (t_ci(in) > 1) {
        // plaintext (tap, d, input ciphertext j, output ciphertext g): on the valid output positions of block b the
        // weight from input channel j ci + (b + d) mod ci to output channel g ci + b, zero where either does not exist
        const uint32_t ci = t_ci(in), per_in = (uint32_t)t_per(in), per_out = (OC + ci - 1) / ci;
        if (plan.sums_by_taps) {
            // plaintext (d, input ciphertext j, sum k, output ciphertext g), k running over the filter taps with the
            // unrotated one first: the weight of output block b on block b, but under the input elements -- the slots
            // of the valid outputs moved by the tap's amount, which the rotation of sum k undoes
            const size_t ftaps = plan.sum_taps.size(), rows = (size_t)ci * per_in * per_out, slots = ctx->N / 2;
            std::vector<std::vector<std::vector<uint32_t>>> per_sum(ftaps, std::vector<std::vector<uint32_t>>(ci));
            std::vector<double> vals(ftaps * rows * ci, 0.0);
            for (size_t k = 0; k < ftaps; k++) {
                const uint32_t tp = plan.sum_taps[k];
                const int32_t amount = conv_tap_amount(ctx, in, geom, tp / geom->fw, tp % geom->fw);
                for (uint32_t b = 0; b < ci; b++)
                    for (uint32_t v : masked_same ? tap_slots[tp] : vslots)
                        per_sum[k][b].push_back((uint32_t)(((u64)v + (u64)amount + (u64)b * in->c_stride) % slots));
                for (size_t r = 0; r < rows; r++) {
                    const size_t g_ = r % per_out, j = (r / per_out) % per_in, d = r / per_out / per_in;
                    for (uint32_t b = 0; b < ci; b++) {
                        const size_t ic = j * ci + (b + d) % ci, oc = g_ * ci + b;
                        if (ic < IC && oc < OC) vals[(k * rows + r) * ci + b] = w[((size_t)tp * IC + ic) * OC + oc];
                    }
                }
            }
            // kept as [d][j][sum k][g] (one multiply-accumulate launch forms all sums): the plaintexts of a sum are
            // encoded together -- they share their slot sets -- and copied to their places
            cw.shared = false;
            cw.pt_scale = q_last;
            const size_t pt_words = (size_t)l * n;
            cw.pts = new Temp(ctx, ftaps * rows * pt_words * sizeof(u64));
            Temp stage(ctx, rows * pt_words * sizeof(u64));
            if (!cw.pts->ok() || !stage.ok()) return HISA_ERR_OOM;
            for (size_t k = 0; k < ftaps; k++) {
                TRY(encode_piecewise_batch(ctx, per_sum[k], vals.data() + k * rows * ci, rows, q_last, (int)l, stage.u()));
                for (size_t dj = 0; dj < (size_t)ci * per_in; dj++)
                    HIP_TRY(ctx, hipMemcpyAsync(cw.pts->u() + ((dj * ftaps + k) * per_out) * pt_words, stage.u() + dj * per_out * pt_words,
                                                per_out * pt_words * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream));
            }
            return HISA_OK;
        }
        if (plan.rotate_sums) {
            // plaintext (tap, input ciphertext j, d, output ciphertext g): the same weight, but on block b + d, where
            // the input channel lies (behind the blocks their copy, or cyclically block 0); taps = filter taps here
            const uint32_t npos = plan.wrap > 0 ? 2 * ci : ci;
            const size_t n_pts = taps * per_in * ci * per_out;
            std::vector<std::vector<uint32_t>> sets(npos);
            for (uint32_t pos = 0; pos < npos; pos++)
                for (uint32_t v : vslots) sets[pos].push_back(v + pos * in->c_stride);
            std::vector<double> vals(n_pts * npos, 0.0);
            for (size_t idx = 0; idx < n_pts; idx++) {
                const size_t g_ = idx % per_out, d = (idx / per_out) % ci, j = (idx / per_out / ci) % per_in;
                const size_t tap = idx / per_out / ci / per_in;
                for (uint32_t b = 0; b < ci; b++) {
                    const size_t ic = j * ci + (b + d) % ci, oc = g_ * ci + b;
                    const size_t pos = plan.wrap > 0 ? b + d : (b + d) % ci;
                    if (ic < IC && oc < OC) vals[idx * npos + pos] = w[(tap * IC + ic) * OC + oc];
                }
            }
            if (masked_same) {
                const auto per_tap = block_sets(npos);
                return build_plain_weights(ctx, sets, vals.data(), plan, per_in, ci * per_out, l, q_last, false, cw, &per_tap);
            }
            return build_plain_weights(ctx, sets, vals.data(), plan, per_in, ci * per_out, l, q_last, false, cw);
        }
        const size_t n_pts = taps * per_in * per_out;
        std::vector<std::vector<uint32_t>> sets(ci);
        for (uint32_t b = 0; b < ci; b++)
            for (uint32_t v : vslots) sets[b].push_back(v + b * in->c_stride);
        std::vector<double> vals(n_pts * ci, 0.0);   // one value per (plaintext, block)
        for (size_t idx = 0; idx < n_pts; idx++) {
            const size_t g_ = idx % per_out, j = (idx / per_out) % per_in, td = idx / per_out / per_in;
            const size_t d = td % ci, tap = td / ci;
            for (uint32_t b = 0; b < ci; b++) {
                const size_t ic = j * ci + (b + d) % ci, oc = g_ * ci + b;
                if (ic < IC && oc < OC) vals[idx * ci + b] = w[(tap * IC + ic) * OC + oc];
            }
        }
        if (masked_same) {
            const auto per_tap = block_sets(ci);
            return build_plain_weights(ctx, sets, vals.data(), plan, per_in, per_out, l, q_last, shared, cw, &per_tap);
        }
        return build_plain_weights(ctx, sets, vals.data(), plan, per_in, per_out, l, q_last, shared, cw);
    }
    if (geom->mode == HISA_CONV_PLAIN)   // plaintext (tap, ic, oc) = weight on every valid output position, zero elsewhere
        return build_plain_weights(ctx, {vslots}, w, plan, IC, OC, l, q_last, shared, cw);
    cw.w_scale = geom->mode == HISA_CONV_MASKED ? q_last / HISA_MASK_SCALE : q_last;
    std::vector<int64_t> w_int(T * OC);
    for (size_t i = 0; i < T * OC; i++) {
        const double v = w[i] * cw.w_scale;
        if (!(fabs(v) < 9.2e18)) return fail(ctx, HISA_ERR_ARG, "weight %g does not fit the fixed-point range", w[i]);
        w_int[i] = (int64_t)round(v);
    }
    TRY(build_scalar_weights(ctx, w_int.data(), plan, IC, OC, l, shared, cw));
    if (geom->mode == HISA_CONV_MASKED) {
        cw.mask = new Temp(ctx, (size_t)l * n * sizeof(u64));
        if (!cw.mask->ok()) return HISA_ERR_OOM;
        std::vector<double> ones(vslots.size(), 1.0);
        TRY(encode_sparse_batch(ctx, vslots, ones.data(), 1, HISA_MASK_SCALE, (int)l, cw.mask->u()));
        cw.pt_scale = HISA_MASK_SCALE;
    }
    return HISA_OK;
}

// the same from fixed-point inputs (what the oracle derived): w_int[T][OC], or plaintext coefficients
static int conv_build_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* w_int, double w_scale, const int64_t* pt_coeffs,
                            double pt_scale, uint32_t OC, const hisa_conv_geom* geom, const ConvPlan& plan, ConvWeights& cw) {
    const uint32_t l = in->cts[0]->limbs, ICm = (uint32_t)t_per(in), OCm = (OC + t_ci(in) - 1) / t_ci(in);
    const size_t n = ctx->N, T = plan.steps.size() * ICm;
    bool shared;
    TRY(conv_wants_shared(ctx, geom, plan, &shared));
    cw.w_scale = w_scale; cw.pt_scale = pt_scale; cw.shared = shared;
    if (geom->mode == HISA_CONV_PLAIN) {
        if (!pt_coeffs) return fail(ctx, HISA_ERR_ARG, "PLAIN mode needs plaintext coefficients");
        cw.w_scale = 1.0;
        if (plan.sums_by_taps) {
            // given as [tap][d][j][g][N]; kept as [d][j][sum k][g][N], the unrotated tap first
            const size_t ci = t_ci(in), ftaps = plan.sum_taps.size();
            std::vector<int64_t> perm(ftaps * ci * ICm * OCm * n);
            for (size_t k = 0; k < ftaps; k++)
                for (size_t dj = 0; dj < ci * ICm; dj++)
                    memcpy(perm.data() + ((dj * ftaps + k) * OCm) * n, pt_coeffs + (((size_t)plan.sum_taps[k] * ci * ICm + dj) * OCm) * n,
                           OCm * n * sizeof(int64_t));
            cw.pts = new Temp(ctx, perm.size() * l * sizeof(u64));
            if (!cw.pts->ok()) return HISA_ERR_OOM;
            return coeffs_to_plain_batch(ctx, perm.data(), perm.size() / n, (int)l, cw.pts->u());
        }
        if (plan.rotate_sums) {
            // given as [tap][d][j][g][N]; the multiply-accumulate reads [tap][j][(d, g)][N]
            const size_t ci = t_ci(in), taps = plan.steps.size();
            std::vector<int64_t> perm(taps * ci * ICm * OCm * n);
            for (size_t tap = 0; tap < taps; tap++)
                for (size_t d = 0; d < ci; d++)
                    for (size_t j = 0; j < ICm; j++)
                        memcpy(perm.data() + (((tap * ICm + j) * ci + d) * OCm) * n,
                               pt_coeffs + (((tap * ci + d) * ICm + j) * OCm) * n, OCm * n * sizeof(int64_t));
            cw.pts = new Temp(ctx, perm.size() * l * sizeof(u64));
            if (!cw.pts->ok()) return HISA_ERR_OOM;
            return coeffs_to_plain_batch(ctx, perm.data(), perm.size() / n, (int)l, cw.pts->u());
        }
        if (!shared) {
            cw.pts = new Temp(ctx, T * OCm * l * n * sizeof(u64));
            if (!cw.pts->ok()) return HISA_ERR_OOM;
            return coeffs_to_plain_batch(ctx, pt_coeffs, T * OCm, (int)l, cw.pts->u());
        }
        const TapSplit ts = split_taps(plan);
        const std::vector<int64_t> cr = pick_taps(pt_coeffs, ts.rot, ICm, OCm * n), cz = pick_taps(pt_coeffs, ts.zero, ICm, OCm * n);
        cw.pts = new Temp(ctx, ts.rot.size() * ICm * OCm * (l + ctx->K) * n * sizeof(u64));
        if (!cw.pts->ok()) return HISA_ERR_OOM;
        TRY(coeffs_to_plain_batch(ctx, cr.data(), ts.rot.size() * ICm * OCm, (int)l, cw.pts->u(), true));
        if (!ts.zero.empty()) {
            cw.pts_zero = new Temp(ctx, ts.zero.size() * ICm * OCm * l * n * sizeof(u64));
            if (!cw.pts_zero->ok()) return HISA_ERR_OOM;
            TRY(coeffs_to_plain_batch(ctx, cz.data(), ts.zero.size() * ICm * OCm, (int)l, cw.pts_zero->u()));
        }
        return HISA_OK;
    }
    if (!w_int) return fail(ctx, HISA_ERR_ARG, "null weights");
    TRY(build_scalar_weights(ctx, w_int, plan, ICm, OC, l, shared, cw));
    if (geom->mode == HISA_CONV_MASKED) {
        if (!pt_coeffs) return fail(ctx, HISA_ERR_ARG, "MASKED mode needs the mask plaintext");
        cw.mask = new Temp(ctx, (size_t)l * n * sizeof(u64));
        if (!cw.mask->ok()) return HISA_ERR_OOM;
        TRY(coeffs_to_plain_batch(ctx, pt_coeffs, 1, (int)l, cw.mask->u()));
    } else {
        cw.pt_scale = 1.0;
    }
    return HISA_OK;
}

// One multiply-accumulate launch of the shared-ModDown convolution: scalar weights (dw) or plaintexts (pts).
// entry_polys / entry_limbs describe the entries read and written; q_only: weights' first l limbs only (dw built on the
// l + K limbs of the accumulators, or plaintexts stored with pt_limbs limbs).
static hipError_t shared_mac(hisa_ctx* ctx, MacArgs ma, const DevWeights* dw, const u64* pts, uint32_t pt_limbs, int batch) {
    if (pts) {
        ma.w = pts; ma.w_stride_t = (u64)ma.OC; ma.w_stride_oc = 1; ma.w_words = (u64)pt_limbs * ctx->N;
        return launch_plain_mac_fp(ctx, ctx->tabs.fprimes, ma, batch, (int)ctx->log_n, ctx->stream);
    }
    if (dw->mfma) {
        u64 qmax = 0;
        for (int k = 0; k < ma.l; k++) qmax = std::max(qmax, ctx->mod[(ma.lq && k >= ma.lq) ? k + ma.gap : k]);
        const int db = qmax < ((u64)1 << 46) ? 6 : 7;
        return launch_scalar_mac_mfma(ctx, ctx->tabs.fprimes, ma, (const int8_t*)dw->digits.blk->ptr, (int)dw->K, (int)dw->K_pad,
                                      (int)dw->OC_pad, dw->c3.as<double>(), dw->da, db, batch, (int)ctx->log_n, ctx->stream);
    }
    return launch_scalar_mac_fp(ctx, ctx->tabs.fprimes, ma, dw->resf.as<double>(), batch, (int)ctx->log_n, ctx->stream);
}

// The convolution with ONE division by P per output ciphertext (the rotations of a convolution are only ever used
// inside its sums): the inputs' c1 is decomposed and raised once, every rotated tap contributes its key-switch
// accumulators -- on l + K limbs, before the division -- times its weight taken on those limbs (E), and sigma(c0)
// times the weight on the l limbs (Q0); unrotated taps contribute weight * (c0, c1) (Z); out = ModDown(E) + (Z0 + Q0,
// Z1), then the mask (MASKED) and the divScalar as usual.  Same result as conv_run up to the rounding of the division.
static int conv_run_shared(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, const ConvPlan& plan, uint32_t OC,
                           const ConvWeights& cw, hisa_tensor* out) {
    const uint32_t B = in->batch, ci = t_ci(in), IC = (uint32_t)t_per(in), OCm = (OC + ci - 1) / ci, l = in->cts[0]->limbs;
    const uint32_t K = ctx->K, le = l + K;
    const size_t nct = (size_t)B * IC, n = ctx->N, n_out = (size_t)B * OCm;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "conv needs a level to rescale into");
    const bool plain = g->mode == HISA_CONV_PLAIN;
    const TapSplit ts = split_taps(plan);
    const size_t S = ts.rot.size();
    if (S == 0 || S > MAX_TAPS || ts.zero.size() > MAX_TAPS) return fail(ctx, HISA_ERR_ARG, "bad tap count");
    std::vector<hisa_ct*> wrapped;
    hisa_ct* const* src = in->cts;
    if (plan.wrap > 0) {
        wrapped.assign(nct, nullptr);
        TRY(hisa_rot_left_batch(ctx, (const hisa_ct* const*)in->cts, nct, norm_step(ctx, -plan.wrap), wrapped.data()));
        BatchIn orig;
        int rcw = gather_batch(ctx, (const hisa_ct* const*)in->cts, nct, &orig);
        if (rcw == HISA_OK) {
            const u64 words = ct_words(ctx, 2, l);
            hipError_t e = launch_addsub(ctx->d_primes, wrapped[0]->data, orig.base, wrapped[0]->data, OP_ADD, (int)l, 2, 2, nct, words,
                                         orig.stride, words, (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rcw = fail(ctx, HISA_ERR_HIP, "conv wrap: %s", hipGetErrorString(e));
        }
        dev_release(ctx, orig.tmp);
        if (rcw != HISA_OK) { free_handles(ctx, wrapped); return rcw; }
        src = wrapped.data();
    }
    BatchIn bi;
    int rc = gather_batch(ctx, (const hisa_ct* const*)src, nct, &bi);
    const u64 acc_bs = (u64)2 * le * n, lw = (u64)l * n;
    // scalar weights: sigma(c0) enters the first accumulators times P (rotation_accumulators_fp), so the weighted sum
    // of the accumulators is all there is; plaintext weights keep sigma(c0) apart (it rides along in their one pass
    // over the plaintexts, on l limbs instead of l + K)
    const bool fold_c0 = !plain;
    Temp acc(ctx, S * nct * acc_bs * sizeof(u64));      // [S][nct][2][l + K][N]
    Temp r0(ctx, (fold_c0 ? 1 : S * nct * lw) * sizeof(u64));   // sigma(c0): [S][nct][l][N]
    Temp E(ctx, n_out * acc_bs * sizeof(u64)), Q0(ctx, n_out * lw * sizeof(u64)), Z(ctx, n_out * 2 * lw * sizeof(u64));
    std::vector<hisa_ct*> outs(n_out, nullptr);
    if (rc == HISA_OK && !(acc.ok() && r0.ok() && E.ok() && Q0.ok() && Z.ok())) rc = HISA_ERR_OOM;
    std::vector<int32_t> rot_steps;
    for (int t : ts.rot) rot_steps.push_back(plan.steps[t]);
    if (rc == HISA_OK) rc = rotation_accumulators_fp(ctx, bi.base, bi.stride, nct, (int)l, rot_steps.data(), (int)S, acc.u(), fold_c0);
    if (!fold_c0) {   // sigma(c0) for every rotated tap, as many taps per launch as the grid allows
        const size_t per_launch = std::max<size_t>(1, std::min<size_t>(GALOIS_TAB_MAX, 65535 / nct));
        for (size_t k0 = 0; k0 < S && rc == HISA_OK; k0 += per_launch) {
            const size_t cnt = std::min(per_launch, S - k0);
            GaloisTab tab = {};
            for (size_t k = 0; k < cnt && rc == HISA_OK; k++) {
                uint64_t gal = 0;
                rc = hisa_galois_elt(ctx, rot_steps[k0 + k], &gal);
                tab.g[k] = (uint32_t)gal;
            }
            if (rc != HISA_OK) break;
            hipError_t e = launch_automorph_steps(bi.base, bi.stride, r0.u() + k0 * nct * lw, lw, tab, (int)cnt, (int)l, nct,
                                                  (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "conv automorphism: %s", hipGetErrorString(e));
        }
    }
    const double mac_scale = in->cts[0]->scale * (plain ? cw.pt_scale : cw.w_scale);
    // scalar weights, no masking multiply in between: the division by P and the divScalar as one division
    // (hisa_set_fused_rescale)
    const bool one_division = ctx->fused_rescale && g->mode == HISA_CONV_SCALAR;
    if (rc == HISA_OK)
        rc = alloc_ct_batch(ctx, n_out, 2, one_division ? l - 1 : l, one_division ? mac_scale / (double)ctx->mod[l - 1] : mac_scale,
                            outs.data());
    if (rc == HISA_OK) {
        hipError_t e;
        MacArgs ma = {};
        ma.IC = (int)IC; ma.OC = (int)OCm;
        // E: the accumulators times the weights on the l + K limbs
        ma.n_taps = (int)S; ma.l = (int)le; ma.ct_words = acc_bs; ma.polys = 2; ma.lq = (int)l; ma.gap = (int)(ctx->L - l);
        for (size_t k = 0; k < S; k++) ma.tap_base[k] = acc.u() + k * nct * acc_bs;
        ma.out = E.u();
        if (plain) {   // the plaintexts are read once: sigma(c0) rides along on the limbs below l (Q0)
            ma.x2 = r0.u(); ma.x2_tap_words = nct * lw; ma.x2_words = lw; ma.out2 = Q0.u();
        }
        e = shared_mac(ctx, ma, cw.dw, plain ? cw.pts->u() : nullptr, le, (int)B);
        ma.x2 = nullptr; ma.out2 = nullptr;
        // Z: the unrotated taps
        if (e == hipSuccess) {
            if (ts.zero.empty()) {
                e = hipMemsetAsync(Z.u(), 0, n_out * 2 * lw * sizeof(u64), ctx->stream);
            } else {
                // (every field the launches above changed is set again: with plaintext weights the Q0 block is skipped)
                ma.n_taps = (int)ts.zero.size(); ma.l = (int)l; ma.ct_words = 2 * lw; ma.polys = 2; ma.lq = 0; ma.gap = 0;
                ma.x2 = nullptr; ma.out2 = nullptr;
                for (size_t k = 0; k < ts.zero.size(); k++) ma.tap_base[k] = bi.base;
                ma.out = Z.u();
                e = shared_mac(ctx, ma, cw.dw_zero, plain ? cw.pts_zero->u() : nullptr, l, (int)B);
            }
        }
        if (e == hipSuccess && plain)   // Z0 += Q0
            e = launch_addsub(ctx->d_primes, Z.u(), Q0.u(), Z.u(), OP_ADD, (int)l, 1, 1, n_out, 2 * lw, lw, 2 * lw, (int)ctx->log_n,
                              ctx->stream);
        if (e != hipSuccess) rc = mac_fail(ctx, e, "conv");
    }
    if (rc == HISA_OK && one_division) rc = moddown_rescale_fp(ctx, E.u(), n_out, (int)l, Z.u(), 2 * lw, 2, outs[0]->data);
    else if (rc == HISA_OK) rc = moddown_add_fp(ctx, E.u(), n_out, (int)l, Z.u(), 2 * lw, 2, 0, outs[0]->data);
    if (rc == HISA_OK && g->mode == HISA_CONV_MASKED) {
        hipError_t e = launch_mul_plain(ctx->d_primes, outs[0]->data, cw.mask->u(), outs[0]->data, (int)l, 2, n_out, 2 * lw, 2 * lw,
                                        (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "conv mask: %s", hipGetErrorString(e));
        for (hisa_ct* c : outs) c->scale = mac_scale * cw.pt_scale;
    }
    dev_release(ctx, bi.tmp);
    free_handles(ctx, wrapped);
    if (rc == HISA_OK && !one_division) rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    if (rc == HISA_OK && one_division && t_analysis) TALLY(rescale, HISA_OP_RESCALE, n_out, l);
    if (rc != HISA_OK) {
        free_handles(ctx, outs);
        return rc;
    }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    const bool keeps_zeros = g->fh == 1 && g->fw == 1 && g->stride == 1 && in->clean;
    fill_out_meta(out, B, OC, plan.out_h, plan.out_w, in->h_stride * g->stride, in->w_stride * g->stride, in->offset,
                  (g->mode != HISA_CONV_SCALAR || keeps_zeros) ? 1u : 0u, ci, in->c_stride);
    return HISA_OK;
}

static int conv_dispatch(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* g, const ConvPlan& plan, uint32_t OC,
                         const ConvWeights& cw, hisa_tensor* out, const RotatedInputs* shared = nullptr) {
    if (plan.rotate_sums)
        return conv_run_sums(ctx, in, g, plan, OC, cw.pts ? cw.pts->u() : nullptr, cw.pt_scale, out, cw.pt_count, cw.pt_packed,
                             shared);
    if (cw.shared) return conv_run_shared(ctx, in, g, plan, OC, cw, out);   // rotates inside its own key switch
    const u64* d_pts = g->mode == HISA_CONV_MASKED ? (cw.mask ? cw.mask->u() : nullptr) : (cw.pts ? cw.pts->u() : nullptr);
    return conv_run(ctx, in, g, plan, OC, cw.dw, cw.w_scale, d_pts, cw.pt_scale, out, cw.pt_count, cw.pt_packed, shared);
}

extern "C" int hisa_conv2d_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* w_int, double w_scale,
                                 const int64_t* pt_coeffs, double pt_scale, uint32_t OC, const hisa_conv_geom* geom,
                                 hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || OC == 0) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    ConvPlan plan;
    TRY(conv_plan(ctx, in, geom, &plan));
    ConvWeights cw;
    TRY(conv_build_fixed(ctx, in, w_int, w_scale, pt_coeffs, pt_scale, OC, geom, plan, cw));
    return conv_dispatch(ctx, in, geom, plan, OC, cw, out);
}

extern "C" int hisa_conv2d(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t OC, const hisa_conv_geom* geom,
                           hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!w || !out || !out->cts || OC == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    ConvPlan plan;
    TRY(conv_plan(ctx, in, geom, &plan));
    ConvWeights cw;
    TRY(conv_build(ctx, in, w, OC, geom, plan, cw));
    return conv_dispatch(ctx, in, geom, plan, OC, cw, out);
}

// The plaintexts of a plan are written once and read at every application, and those reads bound the multiply-accumulate
// launch: they are kept limb-major and, where the primes allow (below 2^48), with six bytes per residue.  (A direct
// call reads its plaintexts once either way, so it keeps the words the encoder wrote.)
static int pack_plain_weights(hisa_ctx* ctx, ConvWeights& cw, uint32_t l) {
    if (!ctx->tabs.fp_ok || !cw.pts || cw.shared || cw.pt_count || l < 1) return HISA_OK;
    const u64 lim = (u64)1 << 48, n = ctx->N, words = (u64)l * n;
    int packed = ctx->mod[0] < lim ? 1 : 0;
    bool rest = l > 1;
    for (uint32_t k = 1; k < l; k++) rest = rest && ctx->mod[k] < lim;
    if (rest) packed |= 2;
    if (cw.pts->blk->bytes % (words * sizeof(u64))) return HISA_OK;
    const u64 cnt = cw.pts->blk->bytes / (words * sizeof(u64));
    const u64 bytes = (((packed & 1) ? 6 : 8) + (u64)(l - 1) * ((packed & 2) ? 6 : 8)) * n * cnt;
    Temp* dst = new Temp(ctx, bytes);
    if (!dst->ok()) { delete dst; return HISA_ERR_OOM; }
    for (u64 c0 = 0; c0 < cnt; c0 += 32768) {
        const u64 c = std::min<u64>(32768, cnt - c0);
        hipLaunchKernelGGL(pack_plain_kernel, dim3((unsigned)(n / NT), l, (unsigned)c), dim3(NT), 0, ctx->stream,
                           cw.pts->u(), dst->as<char>(), (int)l, packed, cnt, c0, (int)ctx->log_n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) { delete dst; return fail(ctx, HISA_ERR_HIP, "plaintext packing: %s", hipGetErrorString(e)); }
    }
    delete cw.pts;     // stream-ordered: the pool may hand the block out again only to later work on this stream
    cw.pts = dst;
    cw.pt_count = cnt;
    cw.pt_packed = packed;
    return HISA_OK;
}

// A convolution whose weights were converted ahead of time for one input layout and level.
#define HISA_MAGIC_CONVPLAN 0x43565031u
struct hisa_conv_plan {
    uint32_t magic;
    hisa_conv_geom geom;
    uint32_t out_channels, channels, height, width, h_stride, w_stride, offset, clean, limbs, c_inner, c_stride;
    ConvWeights cw;
};

extern "C" int hisa_conv2d_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t OC,
                                   const hisa_conv_geom* geom, hisa_conv_plan** plan_out) {
    if (!ctx || !plan_out || !w || OC == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "plans cannot be prepared during an analysis (no kernel runs)");
    TRY(check_tensor(ctx, like));
    ConvPlan plan;
    TRY(conv_plan(ctx, like, geom, &plan));
    hisa_conv_plan* p = new hisa_conv_plan{HISA_MAGIC_CONVPLAN, *geom, OC, like->channels, like->height, like->width,
                                           like->h_stride, like->w_stride, like->offset, like->clean, like->cts[0]->limbs,
                                           t_ci(like), like->c_stride, {}};
    int rc = conv_build(ctx, like, w, OC, geom, plan, p->cw);
    if (rc == HISA_OK && geom->mode == HISA_CONV_PLAIN) rc = pack_plain_weights(ctx, p->cw, like->cts[0]->limbs);
    if (rc != HISA_OK) { delete p; return rc; }
    *plan_out = p;
    return HISA_OK;
}

extern "C" int hisa_conv_plan_free(hisa_ctx* ctx, hisa_conv_plan* plan) {
    if (!ctx || !plan || plan->magic != HISA_MAGIC_CONVPLAN) return fail(ctx, HISA_ERR_ARG, "not a convolution plan");
    plan->magic = 0;
    delete plan;
    return HISA_OK;
}

static int check_plan_for(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_plan* plan, const hisa_tensor* out) {
    if (!ctx || !plan || plan->magic != HISA_MAGIC_CONVPLAN) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    if (in->channels != plan->channels || in->height != plan->height || in->width != plan->width ||
        in->h_stride != plan->h_stride || in->w_stride != plan->w_stride || in->offset != plan->offset ||
        in->clean != plan->clean || t_ci(in) != plan->c_inner || (t_ci(in) > 1 && in->c_stride != plan->c_stride))
        return fail(ctx, HISA_ERR_ARG, "the plan was prepared for another tensor layout");
    if (in->cts[0]->limbs != plan->limbs)
        return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "the plan was prepared for %u limbs, the tensor has %u", plan->limbs,
                    in->cts[0]->limbs);
    return HISA_OK;
}

extern "C" int hisa_conv2d_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_plan* plan, hisa_tensor* out) {
    TRY(check_plan_for(ctx, in, plan, out));
    ConvPlan cp;
    TRY(conv_plan(ctx, in, &plan->geom, &cp));
    return conv_dispatch(ctx, in, &plan->geom, cp, plan->out_channels, plan->cw, out);
}

extern "C" int hisa_conv2d_apply_multi(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_plan* const* plans, size_t n_plans,
                                       hisa_tensor* const* outs) {
    if (!ctx || !plans || !outs || n_plans == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    std::vector<ConvPlan> cps(n_plans);
    for (size_t k = 0; k < n_plans; k++) {
        TRY(check_plan_for(ctx, in, plans[k], outs[k]));
        TRY(conv_plan(ctx, in, &plans[k]->geom, &cps[k]));
    }
    // the plans that rotate their inputs outside a key switch of their own, in the layout of the first such plan,
    // share the rotations by the union of their amounts
    std::vector<int32_t> steps;
    std::vector<char> sharing(n_plans, 0);
    int32_t wrap = -1;
    size_t sharers = 0;
    for (size_t k = 0; k < n_plans; k++) {
        if (plans[k]->cw.shared && !cps[k].rotate_sums) continue;
        if (wrap < 0) wrap = cps[k].wrap;
        if (cps[k].wrap != wrap) continue;
        sharing[k] = 1;
        sharers++;
        steps.insert(steps.end(), cps[k].steps.begin(), cps[k].steps.end());
    }
    RotatedInputs ri;
    const bool share = sharers > 1;
    if (share) TRY(rotate_inputs(ctx, in, wrap, steps, ri));
    int rc = HISA_OK;
    size_t done = 0;
    for (; done < n_plans && rc == HISA_OK; done++)
        rc = conv_dispatch(ctx, in, &plans[done]->geom, cps[done], plans[done]->out_channels, plans[done]->cw, outs[done],
                           share && sharing[done] ? &ri : nullptr);
    if (share) release_inputs(ctx, ri);
    if (rc != HISA_OK)   // the outputs of the plans before the failing one are the caller's no longer
        for (size_t k = 0; k + 1 < done; k++) hisa_tensor_free(ctx, outs[k]);
    return rc;
}

// ---------------------------------------------------------------------------
// fully connected
// ---------------------------------------------------------------------------
// pts: NTT-form plaintexts [OUTC][C][l][N] for outputs o0 .. o0+OUTC-1
static int fc_chunk(hisa_ctx* ctx, const hisa_tensor* in, const BatchIn& bi, const u64* pts, double pt_scale, uint32_t OUTC,
                    hisa_ct** outs) {
    const uint32_t B = in->batch, C = in->channels, l = in->cts[0]->limbs;
    MacArgs ma = {};
    ma.tap_base[0] = bi.base; ma.n_taps = 1; ma.IC = (int)C; ma.OC = (int)OUTC; ma.l = (int)l;
    ma.ct_words = 2 * (u64)l * ctx->N;
    ma.w = pts; ma.w_stride_t = 1; ma.w_stride_oc = C;
    ma.out = outs[0]->data;
    (void)pt_scale;
    const hipError_t e = ctx->tabs.fp_ok ? launch_plain_mac_fp(ctx, ctx->tabs.fprimes, ma, (int)B, (int)ctx->log_n, ctx->stream)
                                         : launch_plain_mac(ctx, ctx->d_primes, ma, (int)B, (int)ctx->log_n, ctx->stream);
    return e == hipSuccess ? HISA_OK : mac_fail(ctx, e, "matmul");
}

static int rotate_add_chain(hisa_ctx* ctx, std::vector<hisa_ct*>& xs, const std::vector<i64>& steps, int sign);

static int fc_finish(hisa_ctx* ctx, const hisa_tensor* in, std::vector<hisa_ct*>& outs, uint32_t OUT, hisa_tensor* out) {
    int rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    // rotate-and-add: after the last step slot `offset` holds the sum over all elements of the plane
    if (rc == HISA_OK) rc = rotate_add_chain(ctx, outs, fc_reduce_steps(ctx, in), 1);
    if (rc != HISA_OK) {
        free_handles(ctx, outs);
        return rc;
    }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    fill_out_meta(out, in->batch, OUT, 1, 1, 1, 1, in->offset, 0);
    return HISA_OK;
}

static int fc_common(hisa_ctx* ctx, const hisa_tensor* in, const double* w, const int64_t* pt_coeffs, double pt_scale,
                     uint32_t OUT, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    TRY(require_hw_tiling(ctx, in, "fc (hisa_matmul reads CHW-tiled tensors)"));
    if (!out || !out->cts || OUT == 0) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    const uint32_t B = in->batch, C = in->channels, l = in->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "fc needs a level to rescale into");
    const size_t n = ctx->N, hw = (size_t)in->height * in->width;
    // the B*OUT accumulators must be one evenly spaced batch; the plaintexts are built OUTC outputs at a time
    const size_t pt_bytes = (size_t)C * l * n * sizeof(u64);
    const uint32_t OUTC = (uint32_t)std::max<size_t>(1, std::min<size_t>(OUT, ((size_t)2 << 30) / pt_bytes));
    BatchIn bi;
    TRY(gather_batch(ctx, (const hisa_ct* const*)in->cts, (size_t)B * C, &bi));
    std::vector<hisa_ct*> outs((size_t)B * OUT, nullptr);
    const double in_scale = in->cts[0]->scale;
    int rc = alloc_ct_batch(ctx, outs.size(), 2, l, in_scale * pt_scale, outs.data());
    const std::vector<uint32_t> slots = plane_slots(in->height, in->width, in->h_stride, in->w_stride, in->offset);
    for (uint32_t o0 = 0; o0 < OUT && rc == HISA_OK; o0 += OUTC) {
        const uint32_t cnt = std::min(OUTC, OUT - o0);
        Temp pts(ctx, (size_t)cnt * pt_bytes);
        if (!pts.ok()) { rc = HISA_ERR_OOM; break; }
        if (w) rc = encode_sparse_batch(ctx, slots, w + (size_t)o0 * C * hw, (size_t)cnt * C, pt_scale, (int)l, pts.u());
        else rc = coeffs_to_plain_batch(ctx, pt_coeffs + (size_t)o0 * C * n, (size_t)cnt * C, (int)l, pts.u());
        if (rc != HISA_OK) break;
        // accumulators of outputs o0.. for every image b: out index b*OUT + o  ->  launch per image
        for (uint32_t b = 0; b < B && rc == HISA_OK; b++) {
            BatchIn one = bi;
            one.base = bi.base + (size_t)b * C * bi.stride;
            hisa_tensor view = *in;
            view.batch = 1;
            rc = fc_chunk(ctx, &view, one, pts.u(), pt_scale, cnt, &outs[(size_t)b * OUT + o0]);
        }
    }
    dev_release(ctx, bi.tmp);
    if (rc != HISA_OK) {
        free_handles(ctx, outs);
        return rc;
    }
    return fc_finish(ctx, in, outs, OUT, out);
}

extern "C" int hisa_fc_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* pt_coeffs, double pt_scale, uint32_t OUT,
                             hisa_tensor* out) {
    if (!pt_coeffs) return fail(ctx, HISA_ERR_ARG, "null plaintext coefficients");
    return fc_common(ctx, in, nullptr, pt_coeffs, pt_scale, OUT, out);
}

extern "C" int hisa_fc(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t OUT, hisa_tensor* out) {
    if (!ctx || !in || !w) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (in->height == 1 && in->width == 1) {
        // Algorithm 1 with a 1x1 filter: conv weights [1][1][IC][OC] = transposed fc weights [OUT][C]
        std::vector<double> wt((size_t)in->channels * OUT);
        for (uint32_t o = 0; o < OUT; o++)
            for (uint32_t c = 0; c < in->channels; c++) wt[(size_t)c * OUT + o] = w[(size_t)o * in->channels + c];
        hisa_conv_geom g = {1, 1, 1, 0, HISA_CONV_SCALAR};
        return hisa_conv2d(ctx, in, wt.data(), OUT, &g, out);
    }
    TRY(check_tensor(ctx, in));
    return fc_common(ctx, in, w, nullptr, (double)ctx->mod[in->cts[0]->limbs - 1], OUT, out);
}

// Weights of a fully connected layer encoded once for a given input layout and level (constants of the circuit:
// the encode, reduction and transform of OUT*C plaintexts is most of the cost of hisa_fc and need not be paid per
// inference).
#define HISA_MAGIC_FCPLAN 0x46435031u
struct hisa_fc_plan {
    uint32_t magic;
    uint32_t out_features, channels, height, width, h_stride, w_stride, offset, limbs;
    double pt_scale;
    DevBlock* pts;   // [OUT][C][limbs][N], NTT form
};

extern "C" int hisa_fc_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t OUT, hisa_fc_plan** plan) {
    if (!ctx || !like || !w || !plan || OUT == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "plans cannot be prepared during an analysis (no kernel runs)");
    TRY(check_tensor(ctx, like));
    TRY(require_hw_tiling(ctx, like, "fc (hisa_matmul reads CHW-tiled tensors)"));
    if (like->height == 1 && like->width == 1)
        return fail(ctx, HISA_ERR_ARG, "a fully connected layer on 1x1 planes multiplies by scalars: nothing to prepare");
    const uint32_t C = like->channels, l = like->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "fc needs a level to rescale into");
    const size_t n = ctx->N, hw = (size_t)like->height * like->width;
    const size_t pt_bytes = (size_t)C * l * n * sizeof(u64);
    DevBlock* blk = dev_alloc(ctx, (size_t)OUT * pt_bytes);
    if (!blk) return HISA_ERR_OOM;
    const double pt_scale = (double)ctx->mod[l - 1];
    const std::vector<uint32_t> slots = plane_slots(like->height, like->width, like->h_stride, like->w_stride, like->offset);
    const uint32_t OUTC = (uint32_t)std::max<size_t>(1, std::min<size_t>(OUT, ((size_t)2 << 30) / pt_bytes));
    int rc = HISA_OK;
    for (uint32_t o0 = 0; o0 < OUT && rc == HISA_OK; o0 += OUTC) {
        const uint32_t cnt = std::min(OUTC, OUT - o0);
        rc = encode_sparse_batch(ctx, slots, w + (size_t)o0 * C * hw, (size_t)cnt * C, pt_scale, (int)l,
                                 (u64*)blk->ptr + (size_t)o0 * C * l * n);
    }
    if (rc != HISA_OK) { dev_release(ctx, blk); return rc; }
    hisa_fc_plan* p = new hisa_fc_plan{HISA_MAGIC_FCPLAN, OUT, C, like->height, like->width, like->h_stride, like->w_stride,
                                       like->offset, l, pt_scale, blk};
    *plan = p;
    return HISA_OK;
}

extern "C" int hisa_fc_plan_free(hisa_ctx* ctx, hisa_fc_plan* plan) {
    if (!ctx || !plan || plan->magic != HISA_MAGIC_FCPLAN) return fail(ctx, HISA_ERR_ARG, "not a fully connected plan");
    dev_release(ctx, plan->pts);
    plan->magic = 0;
    delete plan;
    return HISA_OK;
}

extern "C" int hisa_fc_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_fc_plan* plan, hisa_tensor* out) {
    if (!ctx || !in || !plan || plan->magic != HISA_MAGIC_FCPLAN) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_tensor(ctx, in));
    TRY(require_hw_tiling(ctx, in, "fc (hisa_matmul reads CHW-tiled tensors)"));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    const uint32_t B = in->batch, C = in->channels, l = in->cts[0]->limbs, OUT = plan->out_features;
    if (C != plan->channels || in->height != plan->height || in->width != plan->width || in->h_stride != plan->h_stride ||
        in->w_stride != plan->w_stride || in->offset != plan->offset)
        return fail(ctx, HISA_ERR_ARG, "the plan was prepared for another tensor layout");
    if (l != plan->limbs) return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "the plan was prepared for %u limbs, the tensor has %u",
                                      plan->limbs, l);
    BatchIn bi;
    TRY(gather_batch(ctx, (const hisa_ct* const*)in->cts, (size_t)B * C, &bi));
    std::vector<hisa_ct*> outs((size_t)B * OUT, nullptr);
    int rc = alloc_ct_batch(ctx, outs.size(), 2, l, in->cts[0]->scale * plan->pt_scale, outs.data());
    for (uint32_t b = 0; b < B && rc == HISA_OK; b++) {
        BatchIn one = bi;
        one.base = bi.base + (size_t)b * C * bi.stride;
        hisa_tensor view = *in;
        view.batch = 1;
        rc = fc_chunk(ctx, &view, one, (const u64*)plan->pts->ptr, plan->pt_scale, OUT, &outs[(size_t)b * OUT]);
    }
    dev_release(ctx, bi.tmp);
    if (rc != HISA_OK) {
        free_handles(ctx, outs);
        return rc;
    }
    return fc_finish(ctx, in, outs, OUT, out);
}

// ---------------------------------------------------------------------------
// matmul with replicas (Sec. "Homomorphic Tensor Operations", "Homomorphic matmul" and the CHW paragraph)
// ---------------------------------------------------------------------------
// The element slots of a ciphertext lie inside a block of P slots (P a power of two).  R copies of the block, made
// with log2 R rotations, let one mulPlain serve R outputs, so a layer takes ceil(OUT/R) * (ciphertexts per image)
// multiplications instead of OUT * (ciphertexts per image); the sum inside each block is again a log-step
// rotate-and-add.  Output o = gR + r ends in slot r P + offset of ciphertext g: a CHW-tiled tensor of 1x1 planes.
struct MatmulGeom {
    uint32_t block, R;
    std::vector<i64> replicate;   // rotRight amounts P 2^k
    std::vector<i64> reduce;      // rotLeft amounts
};

static int matmul_geom(hisa_ctx* ctx, const hisa_tensor* in, uint32_t replicas, MatmulGeom* g) {
    if (replicas == 0) return fail(ctx, HISA_ERR_ARG, "replicas must be at least 1");
    const u64 top = t_last(in) + 1, slots = ctx->N / 2;
    u64 block = 1;
    while (block < top) block <<= 1;
    if (block > slots) return fail(ctx, HISA_ERR_ARG, "tensor elements do not fit the slots");
    u64 r = 1;
    while (2 * r <= std::min<u64>(replicas, slots / block)) r *= 2;
    g->block = (uint32_t)block;
    g->R = (uint32_t)r;
    g->replicate.clear();
    for (u64 k = 1; k < r; k <<= 1) g->replicate.push_back((i64)(block * k));
    g->reduce = reduce_steps(in, r > 1 ? block : slots);
    return HISA_OK;
}

extern "C" int hisa_matmul_geometry(hisa_ctx* ctx, const hisa_tensor* in, uint32_t out_features, uint32_t replicas,
                                    uint32_t* block, uint32_t* used_replicas, uint32_t* out_cts) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_layout(ctx, in));
    MatmulGeom g;
    TRY(matmul_geom(ctx, in, replicas, &g));
    if (block) *block = g.block;
    if (used_replicas) *used_replicas = g.R;
    if (out_cts) *out_cts = in->batch * ((out_features + g.R - 1) / g.R);
    return HISA_OK;
}

extern "C" int hisa_matmul_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, uint32_t replicas, int32_t* steps, size_t cap,
                                     size_t* n) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_layout(ctx, in));
    MatmulGeom g;
    TRY(matmul_geom(ctx, in, replicas, &g));
    std::vector<int32_t> all;
    for (const auto& grp : merge_doublings(ctx, g.replicate))
        for (i64 r : grp) all.push_back(norm_step(ctx, -r));
    for (const auto& grp : merge_doublings(ctx, g.reduce))
        for (i64 r : grp) all.push_back(norm_step(ctx, r));
    return write_steps(all, steps, cap, n);
}

// x += rot(x, step) for a batch of ciphertexts, in place
static int rotate_add_batch(hisa_ctx* ctx, std::vector<hisa_ct*>& xs, int32_t step) {
    std::vector<hisa_ct*> rot(xs.size(), nullptr);
    TRY(hisa_rot_left_batch(ctx, (const hisa_ct* const*)xs.data(), xs.size(), step, rot.data()));
    const u64 words = ct_words(ctx, 2, xs[0]->limbs);
    hipError_t e = launch_addsub(ctx->d_primes, xs[0]->data, rot[0]->data, xs[0]->data, OP_ADD, (int)xs[0]->limbs, 2, 2, xs.size(),
                                 words, words, words, (int)ctx->log_n, ctx->stream);
    free_handles(ctx, rot);
    if (e != hipSuccess) return fail(ctx, HISA_ERR_HIP, "rotate-and-add: %s", hipGetErrorString(e));
    return HISA_OK;
}

// A whole rotate-and-add chain over a batch (rotLeft amounts; sign = -1: rotRight): single steps in place, merged
// groups as one sum of rotations of the same ciphertexts (new handles replace xs)
static int rotate_add_chain(hisa_ctx* ctx, std::vector<hisa_ct*>& xs, const std::vector<i64>& steps, int sign) {
    for (const auto& grp : merge_doublings(ctx, steps)) {
        if (grp.size() == 1) {
            TRY(rotate_add_batch(ctx, xs, norm_step(ctx, sign * grp[0])));
            continue;
        }
        const size_t nb = xs.size(), terms = grp.size() + 1;
        std::vector<const hisa_ct*> in(terms * nb);
        std::vector<int32_t> amounts(terms, 0);               // term 0: the ciphertext itself
        for (size_t s = 0; s < terms; s++) {
            if (s) amounts[s] = norm_step(ctx, sign * grp[s - 1]);
            for (size_t b = 0; b < nb; b++) in[s * nb + b] = xs[b];
        }
        std::vector<hisa_ct*> sum(nb, nullptr);
        TRY(hisa_rot_left_sum_batch(ctx, in.data(), nb, amounts.data(), terms, sum.data()));
        free_handles(ctx, xs);
        xs = sum;
    }
    return HISA_OK;
}

// The masking multiply (Sec. "Homomorphic Tensor Operations", SAME-padding paragraph): xs = rescale(in * mask), the
// mask being 0/1 on the element slots at the scale of the last modulus.  masks: NTT-form plaintexts [per][l][N];
// ciphertext j of every image takes mask j (they differ only where a last ciphertext holds fewer channels).
static int mask_run(hisa_ctx* ctx, const hisa_tensor* in, const u64* masks, double mask_scale, std::vector<hisa_ct*>& xs) {
    const uint32_t B = in->batch, per = (uint32_t)t_per(in), l = in->cts[0]->limbs;
    const size_t n_in = (size_t)B * per, n = ctx->N;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "the masking multiply needs a level to rescale into");
    xs.assign(n_in, nullptr);
    BatchIn bi;
    TRY(gather_batch(ctx, (const hisa_ct* const*)in->cts, n_in, &bi));
    const u64 words = ct_words(ctx, 2, l);
    int rc = alloc_ct_batch(ctx, n_in, 2, l, in->cts[0]->scale * mask_scale, xs.data());
    if (rc == HISA_OK) {
        // entry b * per + j takes mask j: one launch
        hipError_t e = launch_mul_plain(ctx->d_primes, bi.base, masks, xs[0]->data, (int)l, 2, n_in, bi.stride, words,
                                        (int)ctx->log_n, ctx->stream, per);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "masking multiply: %s", hipGetErrorString(e));
    }
    dev_release(ctx, bi.tmp);
    if (rc == HISA_OK) rc = hisa_rescale_batch(ctx, xs.data(), n_in);
    if (rc != HISA_OK) free_handles(ctx, xs);
    return rc;
}

// 0/1 masks of the element slots of every ciphertext of an image, NTT form [per][l][N]
static int encode_masks(hisa_ctx* ctx, const hisa_tensor* t, double scale, uint32_t l, u64* out) {
    const uint32_t ci = t_ci(t), per = (uint32_t)t_per(t);
    const size_t hw = (size_t)t->height * t->width;
    std::vector<double> ones((size_t)per * ci * hw, 0.0);
    for (uint32_t j = 0; j < per; j++)
        for (uint32_t c = 0; c < std::min(ci, t->channels - j * ci); c++)
            for (size_t k = 0; k < hw; k++) ones[((size_t)j * ci + c) * hw + k] = 1.0;
    return encode_sparse_batch(ctx, tensor_slots(t), ones.data(), per, scale, (int)l, out);
}

static int mask_finish(hisa_ctx* ctx, const hisa_tensor* in, std::vector<hisa_ct*>& xs, hisa_tensor* out) {
    for (size_t i = 0; i < xs.size(); i++) out->cts[i] = xs[i];
    fill_out_meta(out, in->batch, in->channels, in->height, in->width, in->h_stride, in->w_stride, in->offset, 1, t_ci(in),
                  in->c_stride);
    return HISA_OK;
}

extern "C" int hisa_tensor_mask(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    const uint32_t l = in->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "the masking multiply needs a level to rescale into");
    Temp masks(ctx, t_per(in) * l * ctx->N * sizeof(u64));
    if (!masks.ok()) return HISA_ERR_OOM;
    const double mask_scale = (double)ctx->mod[l - 1];
    TRY(encode_masks(ctx, in, mask_scale, l, masks.u()));
    std::vector<hisa_ct*> xs;
    TRY(mask_run(ctx, in, masks.u(), mask_scale, xs));
    return mask_finish(ctx, in, xs, out);
}

extern "C" int hisa_tensor_mask_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* mask_coeffs, double mask_scale,
                                      hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || !mask_coeffs) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const uint32_t l = in->cts[0]->limbs;
    Temp masks(ctx, t_per(in) * l * ctx->N * sizeof(u64));
    if (!masks.ok()) return HISA_ERR_OOM;
    TRY(coeffs_to_plain_batch(ctx, mask_coeffs, t_per(in), (int)l, masks.u()));
    std::vector<hisa_ct*> xs;
    TRY(mask_run(ctx, in, masks.u(), mask_scale, xs));
    return mask_finish(ctx, in, xs, out);
}

// ---------------------------------------------------------------------------
// bias (not part of Algorithm 1; the HISA's addPlain after a linear layer): channel c's elements get bias[c]
// ---------------------------------------------------------------------------
// pts: [ciphertexts per image][l][N], NTT form, at the ciphertexts' scale; ciphertext b * per + j takes plaintext j
static int bias_run(hisa_ctx* ctx, hisa_tensor* t, const u64* pts) {
    const uint32_t l = t->cts[0]->limbs;
    const size_t per = t_per(t), lw = (size_t)l * ctx->N;
    for (size_t i = 0; i < t_ncts(t); i++) {
        hisa_ct* c = t->cts[i];
        HIP_TRY(ctx, launch_addsub(ctx->d_primes, c->data, pts + (i % per) * lw, c->data, OP_ADD, (int)l, (int)c->polys, 1, 1, 0,
                                   0, 0, (int)ctx->log_n, ctx->stream));
    }
    return HISA_OK;
}

static int bias_check(hisa_ctx* ctx, const hisa_tensor* t) {
    TRY(check_tensor(ctx, t));
    for (size_t i = 1; i < t_ncts(t); i++)
        if (t->cts[i]->scale != t->cts[0]->scale) return fail(ctx, HISA_ERR_SCALE_MISMATCH, "ciphertexts of one tensor at different scales");
    return HISA_OK;
}

extern "C" int hisa_tensor_add_bias(hisa_ctx* ctx, hisa_tensor* t, const double* bias) {
    TRY(bias_check(ctx, t));
    if (!bias) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const uint32_t ci = t_ci(t), per = (uint32_t)t_per(t), l = t->cts[0]->limbs;
    const size_t hw = (size_t)t->height * t->width;
    const double scale = t->cts[0]->scale;
    std::vector<double> vals((size_t)per * ci * hw, 0.0);
    for (uint32_t j = 0; j < per; j++)
        for (uint32_t c = 0; c < std::min(ci, t->channels - j * ci); c++) {
            const double b = bias[(size_t)j * ci + c];
            // the encoder rounds to 64-bit integers: the coefficients of a constant plane stay below |b| * scale
            if (!(fabs(b) * scale < 4.6e18)) return fail(ctx, HISA_ERR_ARG, "bias times scale does not fit 63 bits: rescale first");
            for (size_t k = 0; k < hw; k++) vals[((size_t)j * ci + c) * hw + k] = b;
        }
    Temp pts(ctx, (size_t)per * l * ctx->N * sizeof(u64));
    if (!pts.ok()) return HISA_ERR_OOM;
    TRY(encode_sparse_batch(ctx, tensor_slots(t), vals.data(), per, scale, (int)l, pts.u()));
    return bias_run(ctx, t, pts.u());
}

extern "C" int hisa_tensor_add_bias_fixed(hisa_ctx* ctx, hisa_tensor* t, const int64_t* bias_coeffs) {
    TRY(bias_check(ctx, t));
    if (!bias_coeffs) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const uint32_t l = t->cts[0]->limbs;
    Temp pts(ctx, t_per(t) * l * ctx->N * sizeof(u64));
    if (!pts.ok()) return HISA_ERR_OOM;
    TRY(coeffs_to_plain_batch(ctx, bias_coeffs, t_per(t), (int)l, pts.u()));
    return bias_run(ctx, t, pts.u());
}

// ---------------------------------------------------------------------------
// layout switches (Sec. "Data Layout Selection": layouts that change the tiling around a layer)
// ---------------------------------------------------------------------------
extern "C" int hisa_tensor_layout_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, uint32_t c_inner, uint32_t c_stride,
                                            int32_t* steps, size_t cap, size_t* n) {
    if (!ctx) return HISA_ERR_ARG;
    TRY(check_layout(ctx, in));
    std::vector<int32_t> all;
    if (t_ci(in) > 1) for (uint32_t k = 1; k < t_ci(in); k++) all.push_back(norm_step(ctx, (i64)k * in->c_stride));
    else for (uint32_t k = 1; k < c_inner; k++) all.push_back(norm_step(ctx, -(i64)k * c_stride));
    return write_steps(all, steps, cap, n);
}

// HW -> CHW: channel g c_inner + k moves k blocks to the right and the channels of a group are added up.
extern "C" int hisa_tensor_to_chw(hisa_ctx* ctx, const hisa_tensor* in, uint32_t c_inner, uint32_t c_stride, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || c_inner < 2 || c_stride == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(require_hw_tiling(ctx, in, "the switch to CHW-tiling"));
    if (!in->clean) return fail(ctx, HISA_ERR_ARG, "the switch to CHW-tiling needs a clean tensor (hisa_tensor_mask makes one)");
    hisa_tensor probe = *in;
    probe.c_inner = c_inner; probe.c_stride = c_stride;
    TRY(check_layout(ctx, &probe));
    const uint32_t B = in->batch, C = in->channels, per = (C + c_inner - 1) / c_inner, l = in->cts[0]->limbs;
    const u64 words = ct_words(ctx, 2, l);
    std::vector<hisa_ct*> acc((size_t)B * per, nullptr);
    TRY(alloc_ct_batch(ctx, acc.size(), 2, l, in->cts[0]->scale, acc.data()));
    int rc = HISA_OK;
    // channel k of every group: one batch per k, rotated together and added into the groups' ciphertexts
    for (uint32_t k = 0; k < c_inner && rc == HISA_OK; k++) {
        std::vector<const hisa_ct*> src;
        std::vector<hisa_ct*> dst;
        for (uint32_t b = 0; b < B; b++)
            for (uint32_t g = 0; g < per; g++)
                if (g * c_inner + k < C) { src.push_back(in->cts[(size_t)b * C + g * c_inner + k]); dst.push_back(acc[(size_t)b * per + g]); }
        if (src.empty()) break;
        std::vector<hisa_ct*> rot(src.size(), nullptr);
        rc = hisa_rot_left_batch(ctx, src.data(), src.size(), norm_step(ctx, -(i64)k * c_stride), rot.data());
        for (size_t i = 0; i < src.size() && rc == HISA_OK; i++) {
            hipError_t e = k == 0 ? hipMemcpyAsync(dst[i]->data, rot[i]->data, words * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream)
                                  : launch_addsub(ctx->d_primes, dst[i]->data, rot[i]->data, dst[i]->data, OP_ADD, (int)l, 2, 2, 1, words,
                                                  words, words, (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "layout switch: %s", hipGetErrorString(e));
        }
        free_handles(ctx, rot);
    }
    if (rc != HISA_OK) { free_handles(ctx, acc); return rc; }
    for (size_t i = 0; i < acc.size(); i++) out->cts[i] = acc[i];
    fill_out_meta(out, B, C, in->height, in->width, in->h_stride, in->w_stride, in->offset, 1, c_inner, c_stride);
    return HISA_OK;
}

// CHW -> HW: block k of every ciphertext rotated to the front (the rotations of one ciphertext share its
// decomposition), then everything but the plane masked away.  mask: NTT-form plaintext [l][N].
static int to_hw_run(hisa_ctx* ctx, const hisa_tensor* in, const u64* mask, double mask_scale, hisa_tensor* out) {
    const uint32_t B = in->batch, C = in->channels, ci = t_ci(in), per = (uint32_t)t_per(in), l = in->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "the switch to HW-tiling needs a level to rescale into");
    const size_t n_in = (size_t)B * per;
    const u64 words = ct_words(ctx, 2, l);
    std::vector<int32_t> steps;
    for (uint32_t k = 0; k < ci; k++) steps.push_back(norm_step(ctx, (i64)k * in->c_stride));
    std::vector<hisa_ct*> rot(steps.size() * n_in, nullptr);
    TRY(hisa_rot_left_hoisted_batch(ctx, (const hisa_ct* const*)in->cts, n_in, steps.data(), steps.size(), rot.data()));
    std::vector<hisa_ct*> outs((size_t)B * C, nullptr);
    int rc = alloc_ct_batch(ctx, outs.size(), 2, l, in->cts[0]->scale * mask_scale, outs.data());
    for (uint32_t b = 0; b < B && rc == HISA_OK; b++)
        for (uint32_t c = 0; c < C && rc == HISA_OK; c++) {
            const hisa_ct* src = rot[(size_t)(c % ci) * n_in + (size_t)b * per + c / ci];
            hipError_t e = launch_mul_plain(ctx->d_primes, src->data, mask, outs[(size_t)b * C + c]->data, (int)l, 2, 1, words, words,
                                            (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "layout switch: %s", hipGetErrorString(e));
        }
    free_handles(ctx, rot);
    if (rc == HISA_OK) rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    if (rc != HISA_OK) { free_handles(ctx, outs); return rc; }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    fill_out_meta(out, B, C, in->height, in->width, in->h_stride, in->w_stride, in->offset, 1);
    return HISA_OK;
}

extern "C" int hisa_tensor_to_hw(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    if (t_ci(in) < 2) return fail(ctx, HISA_ERR_ARG, "the tensor is HW-tiled already");
    const uint32_t l = in->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "the switch to HW-tiling needs a level to rescale into");
    Temp mask(ctx, (size_t)l * ctx->N * sizeof(u64));
    if (!mask.ok()) return HISA_ERR_OOM;
    const double mask_scale = (double)ctx->mod[l - 1];
    const std::vector<uint32_t> slots = plane_slots(in->height, in->width, in->h_stride, in->w_stride, in->offset);
    std::vector<double> ones(slots.size(), 1.0);
    TRY(encode_sparse_batch(ctx, slots, ones.data(), 1, mask_scale, (int)l, mask.u()));
    return to_hw_run(ctx, in, mask.u(), mask_scale, out);
}

extern "C" int hisa_tensor_to_hw_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* mask_coeffs, double mask_scale,
                                       hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || !mask_coeffs) return fail(ctx, HISA_ERR_ARG, "bad argument");
    if (t_ci(in) < 2) return fail(ctx, HISA_ERR_ARG, "the tensor is HW-tiled already");
    const uint32_t l = in->cts[0]->limbs;
    Temp mask(ctx, (size_t)l * ctx->N * sizeof(u64));
    if (!mask.ok()) return HISA_ERR_OOM;
    TRY(coeffs_to_plain_batch(ctx, mask_coeffs, 1, (int)l, mask.u()));
    return to_hw_run(ctx, in, mask.u(), mask_scale, out);
}

// masks: NTT-form plaintexts [per][l][N] (needed when R > 1 and the input is not clean), pts: [groups][per][l'][N] with
// l' = l - 1 after the masking multiply, else l.
static int matmul_run(hisa_ctx* ctx, const hisa_tensor* in, const MatmulGeom& g, const u64* masks, double mask_scale,
                      const u64* pts, double pt_scale, uint32_t OUT, hisa_tensor* out) {
    const uint32_t B = in->batch, per = (uint32_t)t_per(in), groups = (OUT + g.R - 1) / g.R;
    uint32_t l = in->cts[0]->limbs;
    const size_t n_in = (size_t)B * per, n = ctx->N;
    const bool masked = g.R > 1 && !in->clean;
    if (l < (masked ? 3u : 2u)) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "matmul needs %d levels to rescale into", masked ? 2 : 1);
    if (masked && !masks) return fail(ctx, HISA_ERR_ARG, "the input is not clean: replicas need the mask");
    std::vector<hisa_ct*> xs;     // working copies of the inputs (R > 1 only)
    int rc = HISA_OK;
    if (g.R > 1) {
        if (masked) {
            rc = mask_run(ctx, in, masks, mask_scale, xs);
            l -= 1;
        } else {
            xs.assign(n_in, nullptr);
            BatchIn bi;
            TRY(gather_batch(ctx, (const hisa_ct* const*)in->cts, n_in, &bi));
            const u64 words = ct_words(ctx, 2, l);
            rc = alloc_ct_batch(ctx, n_in, 2, l, in->cts[0]->scale, xs.data());
            if (rc == HISA_OK) {
                hipError_t e = hipMemcpyAsync(xs[0]->data, bi.base, n_in * words * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream);
                if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "matmul input: %s", hipGetErrorString(e));
            }
            dev_release(ctx, bi.tmp);
        }
        if (rc == HISA_OK) rc = rotate_add_chain(ctx, xs, g.replicate, -1);
        if (rc != HISA_OK) { free_handles(ctx, xs); return rc; }
    }
    hisa_ct* const* src = g.R > 1 ? xs.data() : in->cts;
    std::vector<hisa_ct*> outs((size_t)B * groups, nullptr);
    BatchIn bi;
    rc = gather_batch(ctx, (const hisa_ct* const*)src, n_in, &bi);
    if (rc == HISA_OK) rc = alloc_ct_batch(ctx, outs.size(), 2, l, src[0]->scale * pt_scale, outs.data());
    if (rc == HISA_OK) {
        MacArgs ma = {};
        ma.tap_base[0] = bi.base; ma.n_taps = 1; ma.IC = (int)per; ma.OC = (int)groups; ma.l = (int)l;
        ma.ct_words = 2 * (u64)l * n;
        ma.w = pts; ma.w_stride_t = 1; ma.w_stride_oc = per;
        ma.out = outs[0]->data;
        hipError_t e = ctx->tabs.fp_ok ? launch_plain_mac_fp(ctx, ctx->tabs.fprimes, ma, (int)B, (int)ctx->log_n, ctx->stream)
                                       : launch_plain_mac(ctx, ctx->d_primes, ma, (int)B, (int)ctx->log_n, ctx->stream);
        if (e != hipSuccess) rc = mac_fail(ctx, e, "matmul");
    }
    dev_release(ctx, bi.tmp);
    free_handles(ctx, xs);
    if (rc == HISA_OK) rc = hisa_rescale_batch(ctx, outs.data(), outs.size());
    if (rc == HISA_OK) rc = rotate_add_chain(ctx, outs, g.reduce, 1);
    if (rc != HISA_OK) {
        free_handles(ctx, outs);
        return rc;
    }
    for (size_t i = 0; i < outs.size(); i++) out->cts[i] = outs[i];
    fill_out_meta(out, B, OUT, 1, 1, 1, 1, in->offset, 0, g.R, g.block);
    return HISA_OK;
}

#define HISA_MAGIC_MMPLAN 0x4d4d5031u
struct hisa_matmul_plan {
    uint32_t magic;
    uint32_t out_features, replicas;
    uint32_t channels, height, width, h_stride, w_stride, offset, clean, c_inner, c_stride, limbs;   // built for this input
    double pt_scale, mask_scale;
    DevBlock* pts;     // [groups][per][l'][N]
    DevBlock* masks;   // [per][l][N], or null
};

extern "C" int hisa_matmul_plan_free(hisa_ctx* ctx, hisa_matmul_plan* plan) {
    if (!ctx || !plan || plan->magic != HISA_MAGIC_MMPLAN) return fail(ctx, HISA_ERR_ARG, "not a matmul plan");
    if (plan->pts) dev_release(ctx, plan->pts);
    if (plan->masks) dev_release(ctx, plan->masks);
    plan->magic = 0;
    delete plan;
    return HISA_OK;
}

static hisa_matmul_plan* new_matmul_plan(const hisa_tensor* like, uint32_t OUT, uint32_t replicas) {
    return new hisa_matmul_plan{HISA_MAGIC_MMPLAN, OUT, replicas, like->channels, like->height, like->width, like->h_stride,
                                like->w_stride, like->offset, like->clean, t_ci(like), like->c_stride, like->cts[0]->limbs,
                                1.0, 1.0, nullptr, nullptr};
}

static int matmul_build(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t OUT, uint32_t replicas,
                        hisa_matmul_plan** plan_out) {
    if (!ctx || !w || !plan_out || OUT == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_tensor(ctx, like));
    MatmulGeom g;
    TRY(matmul_geom(ctx, like, replicas, &g));
    const uint32_t ci = t_ci(like), per = (uint32_t)t_per(like), C = like->channels, groups = (OUT + g.R - 1) / g.R;
    uint32_t l = like->cts[0]->limbs;
    const bool masked = g.R > 1 && !like->clean;
    if (l < (masked ? 3u : 2u)) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "matmul needs %d levels to rescale into", masked ? 2 : 1);
    const size_t n = ctx->N, hw = (size_t)like->height * like->width;
    const std::vector<uint32_t> slots = tensor_slots(like);
    hisa_matmul_plan* p = new_matmul_plan(like, OUT, replicas);
    int rc = HISA_OK;
    if (masked) {   // 0/1 on the element slots at the scale of the modulus the divScalar removes: the scale is unchanged
        p->mask_scale = (double)ctx->mod[l - 1];
        p->masks = dev_alloc(ctx, (size_t)per * l * n * sizeof(u64));
        if (!p->masks) rc = HISA_ERR_OOM;
        if (rc == HISA_OK) rc = encode_masks(ctx, like, p->mask_scale, l, (u64*)p->masks->ptr);
        l -= 1;
    }
    if (rc == HISA_OK) {
        p->pt_scale = (double)ctx->mod[l - 1];
        p->pts = dev_alloc(ctx, (size_t)groups * per * l * n * sizeof(u64));
        if (!p->pts) rc = HISA_ERR_OOM;
    }
    if (rc == HISA_OK) {
        // plaintext (g, j): weight of output gR + r and channel j ci + c on element k of the r-th copy
        std::vector<uint32_t> rslots;
        for (uint32_t r = 0; r < g.R; r++)
            for (uint32_t v : slots) rslots.push_back(r * g.block + v);
        const size_t nnz = rslots.size();
        const size_t chunk = std::max<size_t>(1, std::min<size_t>((size_t)groups * per, ((size_t)256 << 20) / (nnz * sizeof(double) + n * 8)));
        std::vector<double> vals;
        for (size_t p0 = 0; p0 < (size_t)groups * per && rc == HISA_OK; p0 += chunk) {
            const size_t cnt = std::min(chunk, (size_t)groups * per - p0);
            vals.assign(cnt * nnz, 0.0);
            for (size_t q = 0; q < cnt; q++) {
                const uint32_t gi = (uint32_t)((p0 + q) / per), j = (uint32_t)((p0 + q) % per);
                for (uint32_t r = 0; r < g.R && gi * g.R + r < OUT; r++)
                    for (uint32_t c = 0; c < std::min(ci, C - j * ci); c++)
                        memcpy(&vals[q * nnz + ((size_t)r * ci + c) * hw], w + ((size_t)(gi * g.R + r) * C + j * ci + c) * hw,
                               hw * sizeof(double));
            }
            rc = encode_sparse_batch(ctx, rslots, vals.data(), cnt, p->pt_scale, (int)l, (u64*)p->pts->ptr + p0 * l * n);
        }
    }
    if (rc != HISA_OK) { hisa_matmul_plan_free(ctx, p); return rc; }
    *plan_out = p;
    return HISA_OK;
}

extern "C" int hisa_matmul_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t OUT, uint32_t replicas,
                                   hisa_matmul_plan** plan_out) {
    if (t_analysis) return fail(ctx, HISA_ERR_ARG, "plans cannot be prepared during an analysis (no kernel runs)");
    return matmul_build(ctx, like, w, OUT, replicas, plan_out);
}

extern "C" int hisa_matmul_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_matmul_plan* plan, hisa_tensor* out) {
    if (!ctx || !plan || plan->magic != HISA_MAGIC_MMPLAN) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    if (in->channels != plan->channels || in->height != plan->height || in->width != plan->width ||
        in->h_stride != plan->h_stride || in->w_stride != plan->w_stride || in->offset != plan->offset ||
        (in->clean != 0) != (plan->clean != 0) || t_ci(in) != plan->c_inner || (t_ci(in) > 1 && in->c_stride != plan->c_stride))
        return fail(ctx, HISA_ERR_ARG, "the plan was prepared for another tensor layout");
    if (in->cts[0]->limbs != plan->limbs)
        return fail(ctx, HISA_ERR_LEVEL_MISMATCH, "the plan was prepared for %u limbs, the tensor has %u", plan->limbs,
                    in->cts[0]->limbs);
    MatmulGeom g;
    TRY(matmul_geom(ctx, in, plan->replicas, &g));
    return matmul_run(ctx, in, g, plan->masks ? (const u64*)plan->masks->ptr : nullptr, plan->mask_scale,
                      (const u64*)plan->pts->ptr, plan->pt_scale, plan->out_features, out);
}

extern "C" int hisa_matmul(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t OUT, uint32_t replicas,
                           hisa_tensor* out) {
    hisa_matmul_plan* plan = nullptr;
    TRY(matmul_build(ctx, in, w, OUT, replicas, &plan));
    const int rc = hisa_matmul_apply(ctx, in, plan, out);
    hisa_matmul_plan_free(ctx, plan);
    return rc;
}

extern "C" int hisa_matmul_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* pt_coeffs, double pt_scale,
                                 const int64_t* mask_coeffs, double mask_scale, uint32_t OUT, uint32_t replicas,
                                 hisa_tensor* out) {
    if (!ctx || !pt_coeffs || OUT == 0) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts) return fail(ctx, HISA_ERR_ARG, "bad output tensor");
    MatmulGeom g;
    TRY(matmul_geom(ctx, in, replicas, &g));
    const uint32_t per = (uint32_t)t_per(in), groups = (OUT + g.R - 1) / g.R;
    uint32_t l = in->cts[0]->limbs;
    const bool masked = g.R > 1 && !in->clean;
    if (masked && !mask_coeffs) return fail(ctx, HISA_ERR_ARG, "the input is not clean: replicas need the mask");
    if (l < (masked ? 3u : 2u)) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "matmul needs %d levels to rescale into", masked ? 2 : 1);
    const size_t n = ctx->N;
    Temp masks(ctx, masked ? (size_t)per * l * n * sizeof(u64) : 8);
    if (!masks.ok()) return HISA_ERR_OOM;
    if (masked) {
        TRY(coeffs_to_plain_batch(ctx, mask_coeffs, per, (int)l, masks.u()));
        l -= 1;
    }
    Temp pts(ctx, (size_t)groups * per * l * n * sizeof(u64));
    if (!pts.ok()) return HISA_ERR_OOM;
    TRY(coeffs_to_plain_batch(ctx, pt_coeffs, (size_t)groups * per, (int)l, pts.u()));
    return matmul_run(ctx, in, g, masked ? masks.u() : nullptr, mask_scale, pts.u(), pt_scale, OUT, out);
}

// ---------------------------------------------------------------------------
// pooling, activation
// ---------------------------------------------------------------------------
extern "C" int hisa_avg_pool2x2(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out) {
    TRY(hisa_sum_pool2x2(ctx, in, out));
    for (size_t i = 0; i < t_ncts(out); i++) out->cts[i]->scale *= 4.0;   // value = polynomial / scale: the mean
    return HISA_OK;
}

extern "C" int hisa_sum_pool2x2(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || in->height < 2 || in->width < 2) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const size_t nct = t_ncts(in);   // every channel of a ciphertext is pooled by the same three rotations
    const uint32_t l = in->cts[0]->limbs;
    const u64 words = ct_words(ctx, 2, l);
    if (ctx->merge_doublings >= 2) {
        // the two-step chain x += rot(x, w_stride); x += rot(x, h_stride) as one sum over the four corners: one
        // decomposition and one division by P per ciphertext (hisa_set_merge_doublings)
        std::vector<const hisa_ct*> terms(4 * nct);
        for (size_t i = 0; i < 4 * nct; i++) terms[i] = in->cts[i % nct];
        const int32_t amounts[4] = {0, norm_step(ctx, (i64)in->w_stride), norm_step(ctx, (i64)in->h_stride),
                                    norm_step(ctx, (i64)in->h_stride + in->w_stride)};
        std::vector<hisa_ct*> sum(nct, nullptr);
        TRY(hisa_rot_left_sum_batch(ctx, terms.data(), nct, amounts, 4, sum.data()));
        for (size_t i = 0; i < nct; i++) out->cts[i] = sum[i];
        fill_out_meta(out, in->batch, in->channels, in->height / 2, in->width / 2, in->h_stride * 2, in->w_stride * 2, in->offset,
                      0, t_ci(in), in->c_stride);
        return HISA_OK;
    }
    std::vector<hisa_ct*> acc(nct, nullptr);
    TRY(alloc_ct_batch(ctx, nct, 2, l, in->cts[0]->scale, acc.data()));
    BatchIn bi;
    int rc = gather_batch(ctx, (const hisa_ct* const*)in->cts, nct, &bi);
    if (rc == HISA_OK) {
        hipError_t e = hipMemcpyAsync(acc[0]->data, bi.base, nct * words * sizeof(u64), hipMemcpyDeviceToDevice, ctx->stream);
        if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "copy: %s", hipGetErrorString(e));
    }
    dev_release(ctx, bi.tmp);
    const i64 shifts[3] = {(i64)in->w_stride, (i64)in->h_stride, (i64)in->h_stride + in->w_stride};
    if (rc == HISA_OK) {   // three rotations of the same inputs share the decomposition of c1
        int32_t steps3[3];
        for (int k = 0; k < 3; k++) steps3[k] = norm_step(ctx, shifts[k]);
        std::vector<hisa_ct*> rot(3 * nct, nullptr);
        rc = hisa_rot_left_hoisted_batch(ctx, (const hisa_ct* const*)in->cts, nct, steps3, 3, rot.data());
        for (int k = 0; k < 3 && rc == HISA_OK; k++) {
            hipError_t e = launch_addsub(ctx->d_primes, acc[0]->data, rot[k * nct]->data, acc[0]->data, OP_ADD, (int)l, 2, 2, nct,
                                         words, words, words, (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "pool add: %s", hipGetErrorString(e));
        }
        if (rc == HISA_OK || rot[0]) free_handles(ctx, rot);
    }
    if (rc != HISA_OK) {
        free_handles(ctx, acc);
        return rc;
    }
    for (size_t i = 0; i < nct; i++) { acc[i]->scale = in->cts[i]->scale; out->cts[i] = acc[i]; }
    fill_out_meta(out, in->batch, in->channels, in->height / 2, in->width / 2, in->h_stride * 2, in->w_stride * 2, in->offset, 0,
                  t_ci(in), in->c_stride);
    return HISA_OK;
}

extern "C" int hisa_poly2_act(hisa_ctx* ctx, const hisa_tensor* in, double a, double b, hisa_tensor* out) {
    TRY(check_tensor(ctx, in));
    if (!out || !out->cts || a == 0.0 || !isfinite(b / a)) return fail(ctx, HISA_ERR_ARG, "bad argument");
    const size_t nct = t_ncts(in);
    const uint32_t l = in->cts[0]->limbs;
    if (l < 2) return fail(ctx, HISA_ERR_DEPTH_EXHAUSTED, "activation needs a level to rescale into");
    std::vector<hisa_ct*> sq(nct, nullptr);
    TRY(hisa_mul_no_relin_batch(ctx, (const hisa_ct* const*)in->cts, (const hisa_ct* const*)in->cts, nct, sq.data()));
    if (ctx->fused_rescale) {
        // the linear term joins (d0, d1) of the unrelinearised square, and the relinearisation's division by P is taken
        // together with the divScalar (hisa_set_fused_rescale)
        const u64 words = ct_words(ctx, 2, l), words3 = ct_words(ctx, 3, l);
        int rc = HISA_OK;
        if (b != 0.0) {
            const double v = (b / a) * in->cts[0]->scale;
            BatchIn bi;
            rc = gather_batch(ctx, (const hisa_ct* const*)in->cts, nct, &bi);
            Temp lin(ctx, nct * words * sizeof(u64));
            if (rc == HISA_OK && !lin.ok()) rc = HISA_ERR_OOM;
            if (rc == HISA_OK) {
                u64 consts[2 * HISA_MAX_PRIMES];
                for (uint32_t i = 0; i < l; i++) {
                    consts[i] = double_to_residue(v, ctx->mod[i]);
                    consts[l + i] = (u64)(((u128)consts[i] << 64) / ctx->mod[i]);
                }
                hipError_t e = launch_mul_const(ctx->d_primes, bi.base, lin.u(), consts, (int)l, (int)(nct * 2), (int)ctx->log_n,
                                                ctx->stream);
                if (e == hipSuccess)   // (d0, d1) += lin: the first two polynomials of every three-polynomial entry
                    e = launch_addsub(ctx->d_primes, sq[0]->data, lin.u(), sq[0]->data, OP_ADD, (int)l, 2, 2, nct, words3, words, words3,
                                      (int)ctx->log_n, ctx->stream);
                if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "activation: %s", hipGetErrorString(e));
            }
            dev_release(ctx, bi.tmp);
        }
        std::vector<hisa_ct*> outs(nct, nullptr);
        if (rc == HISA_OK) rc = alloc_ct_batch(ctx, nct, 2, l - 1, sq[0]->scale / (double)ctx->mod[l - 1], outs.data());
        if (rc == HISA_OK) {
            rc = relinearize_rescale_fp(ctx, sq[0]->data, words3, nct, (int)l, outs[0]->data);
            if (rc != HISA_OK) free_handles(ctx, outs);
        }
        free_handles(ctx, sq);
        if (rc != HISA_OK) return rc;
        for (size_t i = 0; i < nct; i++) out->cts[i] = outs[i];
        fill_out_meta(out, in->batch, in->channels, in->height, in->width, in->h_stride, in->w_stride, in->offset, in->clean,
                      t_ci(in), in->c_stride);
        return HISA_OK;
    }
    int rc = hisa_relinearize_batch(ctx, sq.data(), nct);
    if (rc == HISA_OK && b != 0.0) {
        // (b/a) * x at scale s * s: multiply every residue by round((b/a) * s)
        const double s = in->cts[0]->scale, v = (b / a) * s;
        const u64 words = ct_words(ctx, 2, l);
        BatchIn bi;
        rc = gather_batch(ctx, (const hisa_ct* const*)in->cts, nct, &bi);
        Temp lin(ctx, nct * words * sizeof(u64));
        if (rc == HISA_OK && !lin.ok()) rc = HISA_ERR_OOM;
        if (rc == HISA_OK) {
            u64 consts[2 * HISA_MAX_PRIMES];
            for (uint32_t i = 0; i < l; i++) {
                consts[i] = double_to_residue(v, ctx->mod[i]);
                consts[l + i] = (u64)(((u128)consts[i] << 64) / ctx->mod[i]);
            }
            hipError_t e = launch_mul_const(ctx->d_primes, bi.base, lin.u(), consts, (int)l, (int)(nct * 2), (int)ctx->log_n,
                                            ctx->stream);
            if (e == hipSuccess)
                e = launch_addsub(ctx->d_primes, sq[0]->data, lin.u(), sq[0]->data, OP_ADD, (int)l, 2, 2, nct, words, words, words,
                                  (int)ctx->log_n, ctx->stream);
            if (e != hipSuccess) rc = fail(ctx, HISA_ERR_HIP, "activation: %s", hipGetErrorString(e));
        }
        dev_release(ctx, bi.tmp);
    }
    if (rc == HISA_OK) rc = hisa_rescale_batch(ctx, sq.data(), nct);
    if (rc != HISA_OK) {
        free_handles(ctx, sq);
        return rc;
    }
    for (size_t i = 0; i < nct; i++) out->cts[i] = sq[i];
    fill_out_meta(out, in->batch, in->channels, in->height, in->width, in->h_stride, in->w_stride, in->offset, in->clean,
                  t_ci(in), in->c_stride);
    return HISA_OK;
}

// ---------------------------------------------------------------------------
// tensor <-> host
// ---------------------------------------------------------------------------
extern "C" int hisa_tensor_encrypt(hisa_ctx* ctx, const double* x, double scale, uint32_t limbs, hisa_tensor* t) {
    if (!ctx || !x || limbs < 1 || limbs > ctx->L) return fail(ctx, HISA_ERR_ARG, "bad argument");
    TRY(check_layout(ctx, t));
    const size_t nct = t_ncts(t), n = ctx->N, per = t_per(t), hw = (size_t)t->height * t->width;
    const uint32_t ci = t_ci(t);
    const std::vector<uint32_t> slots = tensor_slots(t);
    {   // the elements of one ciphertext must not share slots
        std::set<uint32_t> uniq(slots.begin(), slots.end());
        if (uniq.size() != slots.size()) return fail(ctx, HISA_ERR_ARG, "tensor elements overlap in the slots");
    }
    // values per ciphertext, channel-major; a last ciphertext with fewer channels is padded with zeros
    std::vector<double> packed;
    const double* values = x;
    if (ci > 1) {
        packed.assign(nct * ci * hw, 0.0);
        for (size_t b = 0; b < t->batch; b++)
            for (size_t c = 0; c < t->channels; c++)
                memcpy(&packed[((b * per + c / ci) * ci + c % ci) * hw], x + (b * t->channels + c) * hw, hw * sizeof(double));
        values = packed.data();
    }
    DevBlock* blk = dev_alloc(ctx, nct * limbs * n * sizeof(u64));
    if (!blk) return HISA_ERR_OOM;
    int rc = encode_sparse_batch(ctx, slots, values, nct, scale, (int)limbs, (u64*)blk->ptr);
    std::vector<hisa_pt*> pts(nct, nullptr);
    if (rc == HISA_OK) {
        blk->refs = (int)nct + 1;
        for (size_t i = 0; i < nct; i++)
            pts[i] = new hisa_pt{HISA_MAGIC_PT, blk, (u64*)blk->ptr + i * limbs * n, limbs, scale};
        rc = hisa_encrypt_batch(ctx, (const hisa_pt* const*)pts.data(), nct, t->cts);
        for (hisa_pt* p : pts) hisa_free(ctx, p);
    }
    dev_release(ctx, blk);
    if (rc == HISA_OK) t->clean = 1;
    return rc;
}

extern "C" int hisa_tensor_decrypt(hisa_ctx* ctx, const hisa_tensor* t, double* x) {
    TRY(check_tensor(ctx, t));
    if (!x) return fail(ctx, HISA_ERR_ARG, "null output");
    const size_t nct = t_ncts(t), per = t_per(t), hw = (size_t)t->height * t->width;
    const uint32_t ci = t_ci(t);
    const std::vector<uint32_t> slots = tensor_slots(t);
    const size_t count = (size_t)*std::max_element(slots.begin(), slots.end()) + 1;
    std::vector<double> re(count);
    for (size_t i = 0; i < nct; i++) {
        hisa_pt* pt = nullptr;
        TRY(hisa_decrypt(ctx, t->cts[i], &pt));
        int rc = hisa_decode(ctx, pt, re.data(), nullptr, count);
        hisa_free(ctx, pt);
        if (rc != HISA_OK) return rc;
        const size_t b = i / per, c0 = (i % per) * ci;
        for (size_t c = c0; c < std::min<size_t>(c0 + ci, t->channels); c++)
            for (size_t k = 0; k < hw; k++) x[(b * t->channels + c) * hw + k] = re[slots[(c - c0) * hw + k]];
    }
    return HISA_OK;
}

extern "C" int hisa_tensor_free(hisa_ctx* ctx, hisa_tensor* t) {
    if (!ctx || !t) return HISA_ERR_ARG;
    if (t->cts)
        for (size_t i = 0; i < t_ncts(t); i++) {
            hisa_free(ctx, t->cts[i]);
            t->cts[i] = nullptr;
        }
    return HISA_OK;
}
