// Single-launch negacyclic NTT / inverse NTT for N = 2^12 .. 2^15 and primes
// below 2^50, with exact fp64 modular arithmetic (fparith.hpp) and the
// neighbouring steps of key switching fused into its load and store stages.
//
// One workgroup transforms one limb-polynomial.  N/32 threads hold 32
// coefficients each in registers (the whole polynomial lives in the register
// file: at N = 2^15 one 1024-thread workgroup fills a CU's registers).  The log2 N
// butterfly levels run as three register-resident radix-32 phases; between
// phases the polynomial is transposed through LDS as two 32-bit halves, so the
// staging buffer is N*4 bytes plus padding (132 KiB at N = 2^15) and the transposes
// need no extra registers.  Global loads and stores are coalesced.
//
// Index bit fields of a coefficient index: idx = (a:5)(b:5)(c:K3), K3 = log2 N - 10
// (the four register mappings are listed at struct Geo).
// Forward (natural in, value at psi^(2 bitrev(i)+1) at index i out): decimation
// in time, levels 1..5 on a (mapping 1), 6..10 on b (2), 11.. on c (3), stores in
// mapping 4.  Inverse: the cyclic inverse transform as decimation in time from
// bit-reversed input (loads in mapping 4, levels on c in 3, then b in 2, then a
// in 1) followed by the untwist psi^-j / N (and an optional extra constant per
// limb).  Only the transpose 1 <-> 2 crosses waves (five workgroup barriers per
// transform); after it the waves run apart and overlap one another's LDS
// traffic, stores and next loads.
#include <cstdio>

#include "hisa_internal.hpp"
#include "fparith.hpp"

template <int K3>
struct Geo {
    static constexpr int LOGN = 10 + K3, TB = 5 + K3, THREADS = 1 << TB, N = 1 << LOGN, CM = (1 << K3) - 1;
    // A coefficient index is (a:5)(b:5)(c:K3), b = (b_high : 5-K3)(b_low : K3).  Four ways to spread the N coefficients
    // over THREADS threads x 32 registers; in each the index is (a term of the thread) | (a compile-time term of the
    // register) with disjoint bits, so addressing needs one register per mapping, not one per element:
    //   1  thread (b, c),      register a             loads/stores of the side whose phase works on a; phase on a
    //   2  thread (a, c),      register b             phase on b
    //   3  thread (a, b_low),  register (b_high, c)   phase on c (2^(5-K3) groups of 2^K3 registers)
    //   4  thread (wave w, lane), register r: index 2048 w + 64 r + lane     coalesced loads/stores
    // In mappings 2, 3 and 4 wave w holds exactly the coefficients [2048 w, 2048 (w+1)), so the transposes between
    // them stay inside a wave and need no workgroup barrier; only 1 <-> 2 crosses waves.
    template <int M> static __device__ __forceinline__ int thread_idx(int t) {
        if (M == 1) return t;
        if (M == 2) return ((t >> K3) << TB) | (t & CM);
        if (M == 3) return ((t >> K3) << TB) | ((t & CM) << K3);
        return ((t >> 6) << 11) | (t & 63);
    }
    template <int M> static constexpr int reg_idx(int r) {
        return M == 1 ? (r << TB) : (M == 2 ? (r << K3) : (M == 3 ? (((r >> K3) << (2 * K3)) | (r & CM)) : (r << 6)));
    }
    // LDS word address of index x: x plus pad words (x >> 5, and one more shift for the small rings) that spread the
    // strided accesses of the mappings over the banks (conflict-free at N = 2^15, at most two-way below).  The
    // shifts act on disjoint bit fields, so the address of (thread | register) is the sum of the two addresses.
    static constexpr int PAD2 = K3 == 3 ? 7 : (K3 == 2 ? 8 : 0);
    static constexpr int LDS_WORDS = N + N / 32 + (PAD2 ? (N >> PAD2) : 0);
    static __device__ __forceinline__ constexpr int lds_of(int x) { return x + (x >> 5) + (PAD2 ? (x >> PAD2) : 0); }
    template <int M> static __device__ __forceinline__ int thread_lds(int t) { return lds_of(thread_idx<M>(t)); }
    template <int M> static constexpr int reg_lds(int r) { return lds_of(reg_idx<M>(r)); }
};

// Read-only tables indexed by wave-uniform values go through the constant address space, which makes the
// compiler use scalar loads (SGPR results, batched, off the vector memory path).  Vector loads of uniform
// addresses were each followed by a wait and cost the kernel dozens of exposed memory latencies.
typedef const __attribute__((address_space(4))) double* cdouble_ptr;
__device__ __forceinline__ cdouble_ptr as_const(const double* p) { return (cdouble_ptr)(unsigned long long)p; }

// Per-lane global accesses go through buffer resources: one (base, size) descriptor per object in scalar registers,
// the lane's byte offset in ONE vector register per mapping and the row's offset in a scalar register or the
// instruction.  Plain pointers cost one or two 64-bit vector additions per access (hundreds per task) and a register
// pair each; this form costs none, and the hardware drops any access beyond `bytes` instead of faulting.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u64 bload(rsrc_t r, uint32_t lane_off, uint32_t row_off) {
    const u32x2_t d = __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, (int)row_off, 0);
    return ((u64)d.y << 32) | d.x;
}
// the same, bypassing the CU's L1 (data that another point in time of this workgroup wrote)
__device__ __forceinline__ u64 bload_glc(rsrc_t r, uint32_t lane_off, uint32_t row_off) {
    const u32x2_t d = __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, (int)row_off, 1);
    return ((u64)d.y << 32) | d.x;
}
__device__ __forceinline__ double bloadf(rsrc_t r, uint32_t lane_off, uint32_t row_off) {
    return __longlong_as_double((long long)bload(r, lane_off, row_off));
}
__device__ __forceinline__ void bstore(rsrc_t r, uint32_t lane_off, uint32_t row_off, u64 x) {
    u32x2_t d;
    d.x = (uint32_t)x; d.y = (uint32_t)(x >> 32);
    __builtin_amdgcn_raw_buffer_store_b64(d, r, (int)lane_off, (int)row_off, 0);
}
__device__ __forceinline__ void bstoref(rsrc_t r, uint32_t lane_off, uint32_t row_off, double x) {
    bstore(r, lane_off, row_off, (u64)__double_as_longlong(x));
}

// keeps the compiler from moving instructions across this point (loads issued in batches stay batches)
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ uint32_t lo32(double v) { return (uint32_t)__double_as_longlong(v); }
__device__ __forceinline__ uint32_t hi32(double v) { return (uint32_t)((u64)__double_as_longlong(v) >> 32); }
__device__ __forceinline__ double mk64(uint32_t lo, uint32_t hi) { return __longlong_as_double((long long)(((u64)hi << 32) | lo)); }

// Synchronisation between the writes and the reads of a transpose.  A transpose inside one wave needs no hardware
// barrier: a wave's LDS instructions execute in issue order, so its reads see its earlier writes and its later
// writes cannot overtake its earlier reads; the compiler only has to keep that order.
template <bool LOCAL>
__device__ __forceinline__ void xchg_sync() {
    if (LOCAL) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }
}

// transpose between two register mappings through LDS, 32-bit halves one after the other
template <int K3, int FROM, int TO, bool LOCAL = false>
__device__ __forceinline__ void exchange(double (&v)[32], uint32_t* lds, int t) {
    typedef Geo<K3> G;
    uint32_t* wr = lds + G::template thread_lds<FROM>(t);
    const uint32_t* rd = lds + G::template thread_lds<TO>(t);
    // the low words are dead once written, so the incoming low words take their registers: 64 live, not 96
    uint32_t lo[32], hi[32];
#pragma unroll
    for (int r = 0; r < 32; r++) { lo[r] = lo32(v[r]); hi[r] = hi32(v[r]); }
#pragma unroll
    for (int r = 0; r < 32; r++) wr[G::template reg_lds<FROM>(r)] = lo[r];
    xchg_sync<LOCAL>();
#pragma unroll
    for (int r = 0; r < 32; r++) lo[r] = rd[G::template reg_lds<TO>(r)];
    xchg_sync<LOCAL>();
#pragma unroll
    for (int r = 0; r < 32; r++) wr[G::template reg_lds<FROM>(r)] = hi[r];
    xchg_sync<LOCAL>();
#pragma unroll
    for (int r = 0; r < 32; r++) hi[r] = rd[G::template reg_lds<TO>(r)];
    xchg_sync<LOCAL>();
#pragma unroll
    for (int r = 0; r < 32; r++) v[r] = mk64(lo[r], hi[r]);
}

// Range: with centred twiddles (|w| <= 0.55 p after a factored product) a level takes max|v| = m p to at most
// (1.21 m + 0.5) p, so five levels from m = 1 (canonical input) stay below 6.2 p and from m = 0.5 (normalised)
// below 5.1 p, inside the 2^53 = 8 * 2^50 that exact integer arithmetic in doubles allows: one normalisation
// per phase is enough and none is needed inside a phase.
__device__ __forceinline__ void bfly(double& x, double& y, double w, double p, double pinv) {
    const double t = fp_mulmod(y, w, p, pinv);
    y = x - t;
    x = x + t;
}

// Twiddles.  The forward twiddle of level j of a phase factors as
//     psi^bitrev(((first + tpart) << j) + g)  =  psi^bitrev((first + tpart) << j)  *  psi^bitrev(g),
// a per-thread value (one per level: five loads per phase, stored at (first << j) + tpart so that lanes read
// consecutive addresses) times a value that is the same for every thread (the first entries of the table, read
// through the scalar cache).  The inverse twiddle psi^(-k N/m), k = (klow << kshift) + tlow, factors the same way.
// The per-thread values are fetched one phase ahead, before the transpose, so that their latency hides behind
// the LDS traffic; the products cost 26 modular multiplications per phase.
template <int BITS, int GROUPS>
__device__ __forceinline__ void load_fwd_tw(double (&bt)[GROUPS][5], rsrc_t tw, int first, const int (&tpart)[GROUPS]) {
#pragma unroll
    for (int grp = 0; grp < GROUPS; grp++)
#pragma unroll
        for (int j = 0; j < BITS; j++) bt[grp][j] = bloadf(tw, (uint32_t)tpart[grp] * 8u, (uint32_t)(first << j) * 8u);
}

// BITS levels over the register-index field of each group of 2^BITS registers (GROUPS groups), largest distance
// first.  UNIFORM: the twiddles depend on the register index only (first phase).
template <int BITS, int GROUPS, int STRIDE, bool UNIFORM>
__device__ __forceinline__ void fwd_phase(double (&v)[32], const double* tw, const double (&bt)[GROUPS][5], double p,
                                          double pinv) {
#pragma unroll
    for (int j = 0; j < BITS; j++) {
        const int half = BITS - 1 - j;
#pragma unroll
        for (int grp = 0; grp < GROUPS; grp++) {
#pragma unroll
            for (int g = 0; g < (1 << j); g++) {
                double w;
                if (UNIFORM) w = as_const(tw)[(1 << j) + g];
                else w = g == 0 ? bt[grp][j] : fp_mulmod(bt[grp][j], as_const(tw)[g], p, pinv);
#pragma unroll
                for (int lo = 0; lo < (1 << half); lo++) {
                    const int r0 = grp * STRIDE + ((g << (half + 1)) | lo);
                    bfly(v[r0], v[r0 + (1 << half)], w, p, pinv);
                }
            }
        }
    }
}

template <int BITS>
__device__ __forceinline__ void load_inv_tw(double (&bt)[5], rsrc_t utw, int t0, int tlow) {
#pragma unroll
    for (int j = 0; j < BITS; j++) bt[j] = bloadf(utw, (uint32_t)tlow * 8u, (8u << (t0 + j)));
}

// Inverse phase (decimation in time from bit-reversed input): level j pairs bit j of the field, smallest distance
// first; twiddle psi^(-k N/2^(t0+j)), k = (klow << t0) + tlow, klow = low j bits of the register field;
// = utw[2^(t0+j) + tlow] * utw[2^j + klow].  UNIFORM: t0 = 0, tlow = 0.
template <int BITS, int GROUPS, int STRIDE, bool UNIFORM>
__device__ __forceinline__ void inv_phase(double (&v)[32], const double* utw, const double (&bt)[5], double p, double pinv) {
#pragma unroll
    for (int j = 0; j < BITS; j++) {
#pragma unroll
        for (int klow = 0; klow < (1 << j); klow++) {
            // The very first level multiplies by 1.  (So does the first group of every later level of this phase, but
            // a butterfly without its product does not reduce y: the values would double per level and leave the
            // exact range after four of them.)
            const bool unit = UNIFORM && j == 0;
            double w = 1.0;
            if (UNIFORM) { if (!unit) w = as_const(utw)[(1 << j) + klow]; }
            else w = klow == 0 ? bt[j] : fp_mulmod(bt[j], as_const(utw)[(1 << j) + klow], p, pinv);
#pragma unroll
            for (int grp = 0; grp < GROUPS; grp++) {
#pragma unroll
                for (int hi = 0; hi < (1 << (BITS - 1 - j)); hi++) {
                    const int r0 = grp * STRIDE + ((hi << (j + 1)) | klow);
                    if (unit) {
                        const double x = v[r0], y = v[r0 + (1 << j)];
                        v[r0] = x + y;
                        v[r0 + (1 << j)] = x - y;
                    } else {
                        bfly(v[r0], v[r0 + (1 << j)], w, p, pinv);
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ uint32_t galois_src_fp(uint32_t i, u64 g, int log_n) {
    const uint32_t mask = (2u << log_n) - 1;
    const uint32_t e = 2 * (__brev(i) >> (32 - log_n)) + 1;
    const uint32_t e2 = (uint32_t)((u64)e * g) & mask;
    return __brev((e2 - 1) >> 1) >> (32 - log_n);
}

// Second launch bound: waves per SIMD the register allocation must leave room for.  N = 2^15 needs 4 (one
// workgroup of 16 waves per CU, 128 registers).  At N = 2^14 the same cap lets two workgroups share a CU and
// overlap one's transposes with the other's arithmetic (measured 16% faster than one workgroup with 256
// registers); at N <= 2^13 the cap costs spills and the 256-register build is the faster one.
#ifndef NTT_FP_MIN_WAVES
#define NTT_FP_MIN_WAVES(K3) ((K3) >= 4 ? 4 : 2)
#endif
template <int K3, int MODE, bool PAIR>
__global__ __launch_bounds__(Geo<K3>::THREADS, NTT_FP_MIN_WAVES(K3)) void ntt_fp_kernel(FpArgs a, FpTask tk) {
    typedef Geo<K3> G;
    extern __shared__ uint32_t lds[];
    const int t = threadIdx.x;
    // Persistent workgroups: each loops over its share of the tasks, so consecutive tasks on a CU run back to back
    // (no dispatch gap, the stores of one overlap the loads of the next).  Workgroups go to the eight XCDs
    // round-robin by id; each XCD gets a contiguous range of tasks, so that tasks sharing inputs (all target
    // limbs of one digit of one ciphertext) run on one XCD at about the same time and find them in its L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    const int per_xcd = (a.n_tasks + 7) >> 3;
    const int task_end = min((xcd + 1) * per_xcd, a.n_tasks);
    constexpr bool INV = (MODE == FP_INV_PLAIN || MODE == FP_INV_TO_Y || MODE == FP_INV_D_TO_Y);
    // The base-conversion modes take the target limbs of a batch entry two at a time: both read the same source
    // digits, so one pass over them forms both sums (half the loads per sum; the loads, not the arithmetic, bound that
    // stage).  The second sum waits in this workgroup's scratch rows (every thread reads back what it wrote itself)
    // while the first is transformed, and is transformed next.
    // PAIR = false: one target limb per task (few source limbs: the loads are not what bounds the stage then, and the
    // round trip of the second sum through the scratch rows costs more than the shared pass saves).
    constexpr bool CONV = (MODE == FP_FWD_CONV || MODE == FP_FWD_CONV_FINAL || MODE == FP_FWD_CONV_SUB);
    constexpr int SUB = (CONV && PAIR) ? 2 : 1;
    const int per_entry = (tk.period + SUB - 1) / SUB;
    // Order of the tasks.  Conversions: entry-major, the target limbs of a batch entry next to one another (they share
    // the entry's source digits).  Plain transforms: limb-major, so that the compute units of an XCD work on one prime
    // at a time and its twiddle tables (as much data as the polynomial itself) stay in that L2.
    const int n_entries = a.n_tasks / per_entry;
    for (int task = xcd * per_xcd + slot; task < task_end; task += slots) {
    const u64 b = CONV ? task / per_entry : task % n_entries;
    const int e_first = CONV ? (task % per_entry) * SUB : task / n_entries;
    for (int half = 0; half < SUB; half++) {
    const int e = e_first + half;
    if (e >= tk.period) break;
    const int pos = tk.pos[e], prime = tk.prime[e];
    const double p = as_const(&a.fprimes[prime].p)[0], pinv = as_const(&a.fprimes[prime].p)[1];
    // Global memory is touched in mapping 1 (lane <-> consecutive coefficients, register r a block of THREADS
    // further) on the side of the transform whose first/last phase works on the top bits, and in mapping 4 on the
    // other side, where the transposes stay inside a wave.
    constexpr int MIN = INV ? 4 : 1;    // mapping of the inverse transform's loads
    constexpr int MOUT = INV ? 1 : 4;   // mapping of the forward transform's stores
    const int t_in = G::template thread_idx<MIN>(t), t_out = G::template thread_idx<MOUT>(t);
    constexpr uint32_t LB = (uint32_t)G::N * 8u;   // bytes of one limb-polynomial
    const uint32_t t8 = (uint32_t)t * 8u, t8_in = (uint32_t)t_in * 8u, t8_out = (uint32_t)t_out * 8u;
    double v[32];

    // ---- load (mapping P1: lane <-> consecutive coefficients; register r holds coefficient r*THREADS + t) ----
    if (MODE == FP_FWD_PLAIN || INV) {
        const rsrc_t src = make_rsrc(a.in + b * a.in_bs + (u64)(pos + a.in_pos_shift) * G::N, LB);
        if (INV && MODE != FP_INV_D_TO_Y && a.galois) {
            // a private copy of the lane id: keeps the 32 gather indices from being kept alive (and spilled) for the
            // address arithmetic of the store stage
            int tg = t_in;
            asm volatile("" : "+v"(tg));
#pragma unroll
            for (int r = 0; r < 32; r++)
                v[r] = fp_from_u64(bload(src, galois_src_fp((uint32_t)(G::template reg_idx<MIN>(r) | tg), a.galois, G::LOGN) * 8u, 0));
        } else if (MODE == FP_INV_D_TO_Y) {
#pragma unroll
            for (int r = 0; r < 32; r++) v[r] = bloadf(src, t8_in, (uint32_t)G::template reg_idx<MIN>(r) * 8u);
        } else if (INV) {
#pragma unroll
            for (int r = 0; r < 32; r++) v[r] = fp_from_u64(bload(src, t8_in, (uint32_t)G::template reg_idx<MIN>(r) * 8u));
        } else {
#pragma unroll
            for (int r = 0; r < 32; r++) v[r] = fp_from_u64(bload(src, t8, (uint32_t)(r << G::TB) * 8u));
        }
    } else {
        // fast base conversion: sum_i y_i * hat_i mod p, y_i centred source digits (already times (D/c_i)^-1), for
        // this limb and (half 0) for its partner, eight rows at a time.  Loads are issued eight at a time, one batch
        // ahead of the arithmetic (two explicit buffers; the fences keep the compiler from sinking each load to its
        // use, which would expose one memory latency per element).
        const rsrc_t scr = make_rsrc(a.scratch + (u64)blockIdx.x * G::N, LB);
        if (half == 0) {
            const int dgi = tk.digit[e];
            const int conv_a = a.dg[dgi].conv_a;
            const double* hat = a.dg[dgi].hat;
            const rsrc_t y = make_rsrc(a.y + b * a.y_bs + (u64)a.dg[dgi].y_pos0 * G::N, (uint32_t)conv_a * LB);
            const bool two = PAIR && e + 1 < tk.period;
            const int prime2 = tk.prime[two ? e + 1 : e];
            const double p2 = as_const(&a.fprimes[prime2].p)[0], pinv2 = as_const(&a.fprimes[prime2].p)[1];
            double bufa[8], bufb[8];
            double* park = (double*)(lds + G::lds_of((t >> 6) << 11)) + (t & 63);   // 16 doubles per lane, lane-interleaved
#pragma unroll
            for (int k = 0; k < 8; k++) bufa[k] = bloadf(y, t8, (uint32_t)(k << G::TB) * 8u);
#pragma unroll
            for (int c = 0; c < 4; c++) {
                double w2[8];
#pragma unroll
                for (int k = 0; k < 8; k++) { v[c * 8 + k] = 0.0; w2[k] = 0.0; }
                // rows 8c .. 8c+7 of source limbs i and i+1 per turn (bufa, then bufb); the batch after the last
                // limb is the first one of the next eight rows
                for (int i = 0; i < conv_a; i += 2) {
                    const bool has1 = i + 1 < conv_a;
                    SCHED_FENCE();
                    {
                        const uint32_t off = has1 ? (uint32_t)(i + 1) * LB + (uint32_t)((c * 8) << G::TB) * 8u
                                                  : (uint32_t)(((c < 3 ? c + 1 : c) * 8) << G::TB) * 8u;
#pragma unroll
                        for (int k = 0; k < 8; k++) bufb[k] = bloadf(y, t8, off + (uint32_t)(k << G::TB) * 8u);
                    }
                    SCHED_FENCE();
                    {
                        const double h1 = as_const(hat)[(u64)i * a.total + prime], h2 = as_const(hat)[(u64)i * a.total + prime2];
#pragma unroll
                        for (int k = 0; k < 8; k++) {
                            v[c * 8 + k] += fp_mulmod(bufa[k], h1, p, pinv);
                            if (PAIR) w2[k] += fp_mulmod(bufa[k], h2, p2, pinv2);
                        }
                    }
                    SCHED_FENCE();
                    {
                        const bool more = i + 2 < conv_a;
                        const uint32_t off = more ? (uint32_t)(i + 2) * LB + (uint32_t)((c * 8) << G::TB) * 8u
                                                  : (uint32_t)(((c < 3 ? c + 1 : c) * 8) << G::TB) * 8u;
                        if (has1) {   // otherwise bufb already holds the first batch of the next rows: hand it over below
#pragma unroll
                            for (int k = 0; k < 8; k++) bufa[k] = bloadf(y, t8, off + (uint32_t)(k << G::TB) * 8u);
                        }
                    }
                    SCHED_FENCE();
                    if (has1) {
                        const double h1 = as_const(hat)[(u64)(i + 1) * a.total + prime],
                                     h2 = as_const(hat)[(u64)(i + 1) * a.total + prime2];
#pragma unroll
                        for (int k = 0; k < 8; k++) {
                            v[c * 8 + k] += fp_mulmod(bufb[k], h1, p, pinv);
                            if (PAIR) w2[k] += fp_mulmod(bufb[k], h2, p2, pinv2);
                        }
                    } else {
#pragma unroll
                        for (int k = 0; k < 8; k++) bufa[k] = bufb[k];
                    }
                    if ((i & 6) == 6) {   // after every eight terms
#pragma unroll
                        for (int k = 0; k < 8; k++) {
                            v[c * 8 + k] = fp_norm(v[c * 8 + k], p, pinv);
                            if (PAIR) w2[k] = fp_norm(w2[k], p2, pinv2);
                        }
                    }
                }
#pragma unroll
                for (int k = 0; k < 8; k++) v[c * 8 + k] = fp_norm(v[c * 8 + k], p, pinv);
                if (two) {
#pragma unroll
                    for (int k = 0; k < 8; k++) bstoref(scr, t8, (uint32_t)((c * 8 + k) << G::TB) * 8u, fp_norm(w2[k], p2, pinv2));
                }
                // Rows 0..15 wait in this wave's own part of the transpose buffer while rows 16..31 are formed: with
                // both sums, their buffers and all 32 rows live the stage would not fit the register file.  The part
                // is free here: the wave is past its last transpose of the previous task, and the workgroup-wide
                // transpose of this one starts behind a barrier that this wave has not reached yet.
                if (PAIR && c == 1) {
#pragma unroll
                    for (int r = 0; r < 16; r++) park[r * 64] = v[r];
                }
            }
            if (PAIR) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                for (int r = 0; r < 16; r++) v[r] = park[r * 64];
            }
        } else {
            // the partner's sum, left in the scratch rows by the step before (read past the L1: the lines may be
            // there from an earlier task)
#pragma unroll
            for (int r = 0; r < 32; r++)
                v[r] = __longlong_as_double((long long)bload_glc(scr, t8, (uint32_t)(r << G::TB) * 8u));
        }
    }

    if (!INV) {
        const double* tw = a.ftw + (u64)prime * G::N;
        const rsrc_t twr = make_rsrc(tw, LB);
        double bt2[1][5];
        {   // levels 1..5 on a: twiddles depend on the register index only
            const double none[1][5] = {};
            fwd_phase<5, 1, 32, true>(v, tw, none, p, pinv);
        }
        {   // per-thread twiddles of levels 6..10 (index 2^(5+j) + a), fetched before the transpose
            const int tp[1] = {t >> K3};
            load_fwd_tw<5, 1>(bt2, twr, 32, tp);
            SCHED_FENCE();
        }
#pragma unroll
        for (int r = 0; r < 32; r++) v[r] = fp_norm(v[r], p, pinv);
        // the waves run apart between the wave-local transposes: all of them must have left the buffer before this
        // workgroup-wide transpose writes to it (its own last barrier guards the other direction)
        __syncthreads();
        exchange<K3, 1, 2>(v, lds, t);
        fwd_phase<5, 1, 32, false>(v, tw, bt2, p, pinv);
        constexpr int GROUPS = 1 << (5 - K3);
        double bt3[GROUPS][5];
        {   // levels 11.. on c: index 2^(10+j) + (a 32 + b), one group per b_high
            int tp[GROUPS];
#pragma unroll
            for (int grp = 0; grp < GROUPS; grp++) tp[grp] = ((t >> K3) << 5) | (grp << K3) | (t & G::CM);
            load_fwd_tw<K3, GROUPS>(bt3, twr, 1024, tp);
            SCHED_FENCE();
        }
#pragma unroll
        for (int r = 0; r < 32; r++) v[r] = fp_norm(v[r], p, pinv);
        exchange<K3, 2, 3, true>(v, lds, t);
        fwd_phase<K3, GROUPS, 1 << K3, false>(v, tw, bt3, p, pinv);
        exchange<K3, 3, MOUT, true>(v, lds, t);
    } else {
        const double* utw = a.utw + (u64)prime * G::N;
        const rsrc_t utwr = make_rsrc(utw, LB);
        double bt[5];
        exchange<K3, MIN, 3, true>(v, lds, t);
        {   // levels t = 0..K3-1 on c
            const double none[5] = {};
            inv_phase<K3, 1 << (5 - K3), 1 << K3, true>(v, utw, none, p, pinv);
        }
        load_inv_tw<5>(bt, utwr, K3, t & G::CM);   // levels K3 + j on b: k = (b mod 2^j) 2^K3 + c
        SCHED_FENCE();
#pragma unroll
        for (int r = 0; r < 32; r++) v[r] = fp_norm(v[r], p, pinv);
        exchange<K3, 3, 2, true>(v, lds, t);
        inv_phase<5, 1, 32, false>(v, utw, bt, p, pinv);
        load_inv_tw<5>(bt, utwr, G::TB, t);        // levels 5 + K3 + j on a: k = (a mod 2^j) 2^(5+K3) + (b, c)
        SCHED_FENCE();
#pragma unroll
        for (int r = 0; r < 32; r++) v[r] = fp_norm(v[r], p, pinv);
        __syncthreads();
        exchange<K3, 2, 1>(v, lds, t);
        inv_phase<5, 1, 32, false>(v, utw, bt, p, pinv);
    }

    // ---- store (mapping P1) ----
    if (MODE == FP_FWD_PLAIN) {
        const rsrc_t dst = make_rsrc(a.out + b * a.out_bs + (u64)pos * G::N, LB);
#pragma unroll
        for (int r = 0; r < 32; r++)
            bstore(dst, t8_out, (uint32_t)G::template reg_idx<MOUT>(r) * 8u, fp_canonical(v[r], p, pinv));
    } else if (MODE == FP_FWD_CONV) {
        // the extended digits stay doubles: their only readers multiply them by key values in the same arithmetic
        const rsrc_t dst = make_rsrc(a.out + b * a.out_bs + (u64)pos * G::N, LB);
#pragma unroll
        for (int r = 0; r < 32; r++)
            bstoref(dst, t8_out, (uint32_t)G::template reg_idx<MOUT>(r) * 8u, fp_norm(v[r], p, pinv));
    } else if (MODE == FP_FWD_CONV_SUB) {
        // out = acc - transform: acc already is (sum * P^-1 + addend), the conversion table carries the P^-1
        const rsrc_t acc = make_rsrc(a.acc + b * a.acc_bs + (u64)(pos + a.acc_pos_shift) * G::N, LB);
        const rsrc_t dst = make_rsrc(a.out + b * a.out_bs + (u64)pos * G::N, LB);
#pragma unroll
        for (int c = 0; c < 4; c++) {
            u64 va[8];
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) va[k] = bload(acc, t8_out, (uint32_t)G::template reg_idx<MOUT>(c * 8 + k) * 8u);
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int r = c * 8 + k;
                bstore(dst, t8_out, (uint32_t)G::template reg_idx<MOUT>(r) * 8u, fp_canonical(fp_from_u64(va[k]) - v[r], p, pinv));
            }
        }
    } else if (MODE == FP_FWD_CONV_FINAL) {
        // out = (acc - conv) * P^-1 (+ addend); operands fetched eight at a time ahead of their use
        const u64* acc_p = a.acc + b * a.acc_bs + (u64)(pos + a.acc_pos_shift) * G::N;
        const rsrc_t acc = make_rsrc(acc_p, LB);
        const rsrc_t dst = make_rsrc(a.out + b * a.out_bs + (u64)pos * G::N, LB);
        const double pin = as_const(a.pinv_tab)[prime];
        const bool with_add = a.add && (int)(b % a.add_div) < a.add_polys;
        const u64 add_ct = a.step_B ? (b / a.add_div) % (u64)a.step_B : b / a.add_div;
        const u64 add_g = a.step_B ? (u64)a.galois_tab[(b / a.add_div) / (u64)a.step_B] : a.add_galois;
        const rsrc_t add = make_rsrc(
            with_add ? a.add + add_ct * a.add_bs + (b % a.add_div) * a.add_ps + (u64)pos * G::N : acc_p, LB);
        int tg = t_out;
        asm volatile("" : "+v"(tg));
#pragma unroll
        for (int c = 0; c < 4; c++) {
            u64 va[8], vb[8];
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int r = c * 8 + k;
                const uint32_t row = (uint32_t)G::template reg_idx<MOUT>(r) * 8u;
                va[k] = bload(acc, t8_out, row);
                if (with_add && add_g)
                    vb[k] = bload(add, galois_src_fp((uint32_t)(G::template reg_idx<MOUT>(r) | tg), add_g, G::LOGN) * 8u, 0);
                else vb[k] = bload(add, t8_out, row);
            }
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int r = c * 8 + k;
                double x = fp_from_u64(va[k]) - fp_norm(v[r], p, pinv);
                x = fp_mulmod(x, pin, p, pinv);
                if (with_add) x += fp_from_u64(vb[k]);
                bstore(dst, t8_out, (uint32_t)G::template reg_idx<MOUT>(r) * 8u, fp_canonical(x, p, pinv));
            }
        }
    } else {
        const rsrc_t vtw = make_rsrc(a.vtw + (u64)prime * G::N, LB);
        const double post = MODE == FP_INV_TO_Y ? as_const(a.post)[e] : 1.0;   // FP_INV_D_TO_Y: the input carries it
        // one of the two outputs is null, according to the mode; its descriptor is then never used
        const rsrc_t dst = make_rsrc(MODE == FP_INV_PLAIN ? (const void*)(a.out + b * a.out_bs + (u64)pos * G::N)
                                                          : (const void*)(a.yout + b * a.yout_bs + (u64)pos * G::N), LB);
#pragma unroll
        for (int c = 0; c < 4; c++) {
            double w8[8];
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) w8[k] = bloadf(vtw, t8, (uint32_t)((c * 8 + k) << G::TB) * 8u);
            SCHED_FENCE();
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const int r = c * 8 + k;
                const double x = fp_mulmod(v[r], w8[k], p, pinv);
                if (MODE == FP_INV_PLAIN) bstore(dst, t8, (uint32_t)(r << G::TB) * 8u, fp_canonical(x, p, pinv));
                else if (MODE == FP_INV_D_TO_Y) bstoref(dst, t8, (uint32_t)(r << G::TB) * 8u, fp_norm(x, p, pinv));
                else bstoref(dst, t8, (uint32_t)(r << G::TB) * 8u, fp_norm(fp_mulmod(x, post, p, pinv), p, pinv));
            }
        }
    }
    }  // the one or two limbs of a task
    }  // task loop
}

template <int K3, int MODE, bool PAIR>
static hipError_t launch_one(const FpArgs& a, const FpTask& tk, u64 n_batch, hipStream_t st) {
    DRY_RUN_RETURN();
    typedef Geo<K3> G;
    static bool attr_set = false;
    const size_t lds_bytes = (size_t)G::LDS_WORDS * 4;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)ntt_fp_kernel<K3, MODE, PAIR>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // the name rocprofv3 prints for this instantiation (PAIR only means something for the conversion modes)
    static char name[40] = "";
    if (!name[0]) snprintf(name, sizeof name, "ntt_fp_kernel<%d, %d, %s>", K3, MODE, PAIR ? "true" : "false");
    ProfScope prof__(name, st);
    FpArgs args = a;
    constexpr bool conv_mode = (MODE == FP_FWD_CONV || MODE == FP_FWD_CONV_FINAL || MODE == FP_FWD_CONV_SUB) && PAIR;   // two target limbs per task
    args.n_tasks = (int)(n_batch * (conv_mode ? (tk.period + 1) / 2 : tk.period));
    static int n_cu = 0;
    if (!n_cu) {
        hipDeviceProp_t prop;
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorInvalidDevice;
        n_cu = prop.multiProcessorCount > 8 ? prop.multiProcessorCount : 8;
    }
    // as many workgroups as are resident on the chip at once
    static int per_cu = 0;
    if (!per_cu) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)ntt_fp_kernel<K3, MODE, PAIR>, G::THREADS, lds_bytes) !=
                hipSuccess || nb < 1)
            nb = 1;
        per_cu = nb;
    }
    unsigned grid = (unsigned)(n_cu * per_cu) & ~7u;
    const unsigned need = (unsigned)((args.n_tasks + 7) / 8) * 8;
    if (grid > need) grid = need;
    if (conv_mode) {   // one scratch polynomial per workgroup
        const unsigned fit = (unsigned)(a.scratch_polys) & ~7u;
        if (fit < 8) return hipErrorInvalidValue;
        if (grid > fit) grid = fit;
    }
    hipLaunchKernelGGL((ntt_fp_kernel<K3, MODE, PAIR>), dim3(grid), dim3(G::THREADS), lds_bytes, st, args, tk);
    return hipGetLastError();
}

// Two target limbs per pass, or one?  A paired task costs r(a) times a single one (a = source limbs: 1.71 at a = 6
// from the tuning harness, falling slowly with more sources, rising with fewer, where the scratch round trip of the
// second sum outweighs the shared loads) and there are half as many; what decides is the number of rounds the chip
// needs for the tasks of the launch.  Measured on batches of 64 at N = 2^15: a = 6 and 16 gain 5-11 % paired, a <= 4
// lose 5-20 %, a = 5 gains with 15 target limbs (2 rounds against 4) and loses with 10 (2 against 3); launches that
// do not fill the chip once are always faster unpaired (twice the parallelism, shorter tasks).
u64 fp_resident_workgroups(int log_n) {
    static int n_cu = 0;
    if (!n_cu) {
        hipDeviceProp_t prop;
        int dev = 0;
        n_cu = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 8)
                   ? prop.multiProcessorCount : 256;
    }
    return (u64)n_cu << (log_n >= 15 ? 0 : 15 - log_n);   // 16 waves a compute unit
}

// estimated time of one conversion launch, in units of one unpaired task, and whether pairing gives it
double fp_conversion_cost(int log_n, int conv_a, int period, u64 n_batch, bool* paired) {
    const u64 resident = fp_resident_workgroups(log_n);
    const u64 rounds_p = (n_batch * (u64)((period + 1) / 2) + resident - 1) / resident;
    const u64 rounds_u = (n_batch * (u64)period + resident - 1) / resident;
    const double r = conv_a >= 6 ? fmax(1.6, 1.71 - 0.01 * (conv_a - 6)) : 1.71 + 0.07 * (6 - conv_a);
    const bool pair = (double)rounds_p * r < (double)rounds_u;
    if (paired) *paired = pair;
    return pair ? (double)rounds_p * r : (double)rounds_u;
}

static bool pair_conversions(int log_n, int conv_a, int period, u64 n_batch) {
    bool pair = false;
    fp_conversion_cost(log_n, conv_a, period, n_batch, &pair);
    return pair;
}

template <int MODE>
static hipError_t dispatch_k3(int log_n, const FpArgs& a, const FpTask& tk, u64 n_batch, hipStream_t st) {
    constexpr bool conv_mode = MODE == FP_FWD_CONV || MODE == FP_FWD_CONV_FINAL || MODE == FP_FWD_CONV_SUB;
    if (conv_mode && (a.no_pair || a.n_digits > 1 || !pair_conversions(log_n, a.conv_a, tk.period, n_batch))) {
        switch (log_n) {
            case 12: return launch_one<2, MODE, !conv_mode>(a, tk, n_batch, st);
            case 13: return launch_one<3, MODE, !conv_mode>(a, tk, n_batch, st);
            case 14: return launch_one<4, MODE, !conv_mode>(a, tk, n_batch, st);
            case 15: return launch_one<5, MODE, !conv_mode>(a, tk, n_batch, st);
            default: return hipErrorInvalidValue;
        }
    }
    switch (log_n) {
        case 12: return launch_one<2, MODE, true>(a, tk, n_batch, st);
        case 13: return launch_one<3, MODE, true>(a, tk, n_batch, st);
        case 14: return launch_one<4, MODE, true>(a, tk, n_batch, st);
        case 15: return launch_one<5, MODE, true>(a, tk, n_batch, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_ntt_fp(int mode, int log_n, const FpArgs& a_in, const FpTask& tk, u64 n_batch, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_batch == 0 || tk.period <= 0) return hipSuccess;
    FpArgs a = a_in;
    if (mode == FP_FWD_CONV || mode == FP_FWD_CONV_FINAL || mode == FP_FWD_CONV_SUB) {
        if (a.n_digits < 0 || a.n_digits > FP_MAX_DIGITS || tk.period > HISA_MAX_PRIMES) return hipErrorInvalidValue;
        if (a.n_digits == 0) {
            a.n_digits = 1;
            a.dg[0].hat = a.hat; a.dg[0].y_pos0 = a.y_pos0; a.dg[0].conv_a = a.conv_a;
        } else {
            // the single-digit fields then describe the first digit (the size checks below read them)
            a.hat = a.dg[0].hat; a.y_pos0 = a.dg[0].y_pos0; a.conv_a = a.dg[0].conv_a;
        }
        for (int d = 0; d < a.n_digits; d++)
            if (!a.dg[d].hat || a.dg[d].conv_a <= 0 || a.dg[d].y_pos0 < 0) return hipErrorInvalidValue;
        for (int e = 0; e < tk.period; e++)
            if (tk.digit[e] < 0 || tk.digit[e] >= a.n_digits) return hipErrorInvalidValue;
    }
    // every pointer a mode dereferences must be set: a missing one is a host error, not a device fault
    if (tk.period > HISA_MAX_PRIMES || !a.fprimes) return hipErrorInvalidValue;
    for (int e = 0; e < tk.period; e++)
        if (tk.prime[e] < 0) return hipErrorInvalidValue;
    const bool inv = mode == FP_INV_PLAIN || mode == FP_INV_TO_Y || mode == FP_INV_D_TO_Y;
    const bool conv = mode == FP_FWD_CONV || mode == FP_FWD_CONV_FINAL || mode == FP_FWD_CONV_SUB;
    if (inv && (!a.in || !a.utw || !a.vtw)) return hipErrorInvalidValue;
    if (!inv && !a.ftw) return hipErrorInvalidValue;
    if (mode == FP_FWD_PLAIN && !a.in) return hipErrorInvalidValue;
    if (mode == FP_INV_TO_Y && (!a.yout || !a.post)) return hipErrorInvalidValue;
    if (mode == FP_INV_D_TO_Y && (!a.yout || a.galois)) return hipErrorInvalidValue;
    if (mode != FP_INV_TO_Y && mode != FP_INV_D_TO_Y && !a.out) return hipErrorInvalidValue;
    if (mode == FP_FWD_CONV_SUB && !a.acc) return hipErrorInvalidValue;
    if (conv && (!a.y || !a.hat || a.conv_a <= 0 || a.total <= 0)) return hipErrorInvalidValue;
    if (conv && !a.no_pair && (!a.scratch || a.scratch_polys < 8)) return hipErrorInvalidValue;
    if (mode == FP_FWD_CONV_FINAL && (!a.acc || !a.pinv_tab || (a.add && a.add_div <= 0))) return hipErrorInvalidValue;
    // rotation-major entries: every entry's rotation index must fall inside galois_tab
    if (mode == FP_FWD_CONV_FINAL && a.add && (a.step_B < 0 ||
        (a.step_B > 0 && (n_batch + (u64)a.add_div * a.step_B - 1) / ((u64)a.add_div * a.step_B) > FP_MAX_STEPS)))
        return hipErrorInvalidValue;
    switch (mode) {
        case FP_FWD_PLAIN: return dispatch_k3<FP_FWD_PLAIN>(log_n, a, tk, n_batch, st);
        case FP_INV_PLAIN: return dispatch_k3<FP_INV_PLAIN>(log_n, a, tk, n_batch, st);
        case FP_INV_TO_Y: return dispatch_k3<FP_INV_TO_Y>(log_n, a, tk, n_batch, st);
        case FP_FWD_CONV: return dispatch_k3<FP_FWD_CONV>(log_n, a, tk, n_batch, st);
        case FP_FWD_CONV_FINAL: return dispatch_k3<FP_FWD_CONV_FINAL>(log_n, a, tk, n_batch, st);
        case FP_INV_D_TO_Y: return dispatch_k3<FP_INV_D_TO_Y>(log_n, a, tk, n_batch, st);
        case FP_FWD_CONV_SUB: return dispatch_k3<FP_FWD_CONV_SUB>(log_n, a, tk, n_batch, st);
        default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------------------
// inner product with the switching key, fp64
// ---------------------------------------------------------------------------
#define IPF_NT 256
#define IPF_ZSPLIT 8
#define IPF_MAXD 8
// One thread owns one coefficient of one extended limb: the 2*digits key values stay in registers while the
// thread walks over its share of the batch, so the key is read IPF_ZSPLIT times per batch (from the L2 after the
// first: see the launch order below), not once per ciphertext.
__global__ __launch_bounds__(IPF_NT) void inner_product_fp_kernel(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits,
                                                                  int l, int K, int L, int alpha, const u64* key, int total,
                                                                  const u64* own_src, u64 own_bs, u64 galois, int gather_ext,
                                                                  u64* acc, u64 acc_bs, u64 n_batch, int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t j = blockIdx.x * IPF_NT + threadIdx.x;
    // the limb is the slowest index of the launch: the blocks that share a limb's key rows (and sit on the same XCD,
    // the number of blocks along x being a multiple of 8) run together and find them in that L2
    const int x = blockIdx.z;
    const int ext_limbs = l + K;
    const int prime = x < l ? x : L + (x - l);
    const int own_digit = x < l ? x / alpha : -1;
    const double p = as_const(&fprimes[prime].p)[0], pinv = as_const(&fprimes[prime].p)[1];
    // own limbs always read through the automorphism; the extended digits too when they were computed from the
    // unrotated polynomial (hoisted rotations: ModUp commutes with the automorphism)
    const uint32_t jsrc = galois ? galois_src_fp(j, galois, log_n) : j;
    const uint32_t jext = gather_ext ? jsrc : j;
    const u64 per = (n_batch + IPF_ZSPLIT - 1) / IPF_ZSPLIT;
    const u64 b0 = (u64)blockIdx.y * per;
    const u64 b1 = b0 + per < n_batch ? b0 + per : n_batch;
    double kb[IPF_MAXD], ka[IPF_MAXD];
#pragma unroll
    for (int d = 0; d < IPF_MAXD; d++) {
        if (d < digits) {
            kb[d] = fp_from_u64(key[(((u64)d * 2 + 0) * total + prime) * n + j]);
            ka[d] = fp_from_u64(key[(((u64)d * 2 + 1) * total + prime) * n + j]);
        }
    }
    for (u64 b = b0; b < b1; b++) {
        double sb = 0.0, sa = 0.0;
#pragma unroll
        for (int d = 0; d < IPF_MAXD; d++) {
            if (d < digits) {
                const double e = d == own_digit ? fp_from_u64(own_src[b * own_bs + (u64)x * n + jsrc])
                                                : ext[b * ext_bs + ((u64)d * ext_limbs + x) * n + jext];
                sb += fp_mulmod(e, kb[d], p, pinv);
                sa += fp_mulmod(e, ka[d], p, pinv);
            }
        }
        acc[b * acc_bs + (u64)x * n + j] = fp_canonical(sb, p, pinv);
        acc[b * acc_bs + ((u64)ext_limbs + x) * n + j] = fp_canonical(sa, p, pinv);
    }
}

// The same inner product with the elementwise ends of the ModDown folded in (struct IpFold): this kernel waits for
// memory, so the extra products cost nothing here, while the transform kernels that would do them wait for the
// vector ALU.  Limbs of q: acc = sum * P^-1 + addend, canonical; special limbs: acc = sum * (P/p_m)^-1, doubles.
__global__ __launch_bounds__(IPF_NT) void inner_product_fold_fp_kernel(const FpPrime* fprimes, const double* ext, u64 ext_bs,
                                                                       int digits, int l, int K, int L, int alpha, const u64* key,
                                                                       int total, const u64* own_src, u64 own_bs, u64 galois,
                                                                       int gather_ext, u64* acc, u64 acc_bs, u64 n_batch,
                                                                       int log_n, IpFold f) {
    const u64 n = (u64)1 << log_n;
    const uint32_t j = blockIdx.x * IPF_NT + threadIdx.x;
    const int x = blockIdx.z;     // limb-slowest launch order, as in inner_product_fp_kernel
    const int ext_limbs = l + K;
    const int prime = x < l ? x : L + (x - l);
    const int own_digit = x < l ? x / alpha : -1;
    const double p = as_const(&fprimes[prime].p)[0], pinv = as_const(&fprimes[prime].p)[1];
    const uint32_t jsrc = galois ? galois_src_fp(j, galois, log_n) : j;
    const uint32_t jext = gather_ext ? jsrc : j;
    const u64 per = (n_batch + IPF_ZSPLIT - 1) / IPF_ZSPLIT;
    const u64 b0 = (u64)blockIdx.y * per;
    const u64 b1 = b0 + per < n_batch ? b0 + per : n_batch;
    const bool special = x >= l;
    const double cst = special ? as_const(f.post_p)[x - l] : as_const(f.pin_tab)[prime];
    const bool add0 = !special && f.add != nullptr && f.add_polys > 0, add1 = !special && f.add != nullptr && f.add_polys > 1;
    double kb[IPF_MAXD], ka[IPF_MAXD];
#pragma unroll
    for (int d = 0; d < IPF_MAXD; d++) {
        if (d < digits) {
            kb[d] = fp_from_u64(key[(((u64)d * 2 + 0) * total + prime) * n + j]);
            ka[d] = fp_from_u64(key[(((u64)d * 2 + 1) * total + prime) * n + j]);
        }
    }
    for (u64 b = b0; b < b1; b++) {
        double sb = 0.0, sa = 0.0;
#pragma unroll
        for (int d = 0; d < IPF_MAXD; d++) {
            if (d < digits) {
                const double e = d == own_digit ? fp_from_u64(own_src[b * own_bs + (u64)x * n + jsrc])
                                                : ext[b * ext_bs + ((u64)d * ext_limbs + x) * n + jext];
                sb += fp_mulmod(e, kb[d], p, pinv);
                sa += fp_mulmod(e, ka[d], p, pinv);
            }
        }
        // |sum| <= 8 * 0.55 p < 2^53: the product with the constant needs no normalisation first
        double rb = fp_mulmod(sb, cst, p, pinv), ra = fp_mulmod(sa, cst, p, pinv);
        u64* dst = acc + b * acc_bs;
        if (special) {
            dst[(u64)x * n + j] = (u64)__double_as_longlong(fp_norm(rb, p, pinv));
            dst[((u64)ext_limbs + x) * n + j] = (u64)__double_as_longlong(fp_norm(ra, p, pinv));
        } else {
            if (add0) rb += fp_from_u64(f.add[b * f.add_bs + (u64)x * n + jsrc]);
            if (add1) ra += fp_from_u64(f.add[b * f.add_bs + f.add_ps + (u64)x * n + jsrc]);
            dst[(u64)x * n + j] = fp_canonical(rb, p, pinv);
            dst[((u64)ext_limbs + x) * n + j] = fp_canonical(ra, p, pinv);
        }
    }
}

// Several rotations of the same ciphertexts: blockIdx.z is the rotation; its key values stay in registers while the
// thread walks over the batch.  The extended digits come from the unrotated polynomial and are gathered through the
// rotation's automorphism like the own-digit limbs.
__global__ __launch_bounds__(IPF_NT) void inner_product_steps_fp_kernel(const FpPrime* fprimes, const double* ext, u64 ext_bs,
                                                                        int digits, int l, int K, int L, int alpha, IpSteps steps,
                                                                        int total, const u64* own_src, u64 own_bs, u64* acc,
                                                                        u64 acc_bs, u64 n_batch, const u64* c0_src,
                                                                        const u64* pmod, int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t j = blockIdx.x * IPF_NT + threadIdx.x;
    // the rotations of a limb run together: they read the same extended digits (through different automorphisms)
    const int x = blockIdx.z, s = blockIdx.y;
    const int ext_limbs = l + K;
    const int prime = x < l ? x : L + (x - l);
    const int own_digit = x < l ? x / alpha : -1;
    const double p = as_const(&fprimes[prime].p)[0], pinv = as_const(&fprimes[prime].p)[1];
    const u64* key = steps.key[s];
    const uint32_t jsrc = galois_src_fp(j, steps.galois[s], log_n);
    double kb[IPF_MAXD], ka[IPF_MAXD];
#pragma unroll
    for (int d = 0; d < IPF_MAXD; d++) {
        if (d < digits) {
            kb[d] = fp_from_u64(key[(((u64)d * 2 + 0) * total + prime) * n + j]);
            ka[d] = fp_from_u64(key[(((u64)d * 2 + 1) * total + prime) * n + j]);
        }
    }
    // c0_src: the first accumulator also takes P * sigma_s(c0) on the limbs of q (what ModDown turns back into
    // sigma_s(c0): the rotated ciphertext is then the ModDown of the accumulators alone)
    const bool fold = c0_src != nullptr && x < l;
    const double pm = fold ? fp_from_u64(pmod[prime]) : 0.0;
    for (u64 b = 0; b < n_batch; b++) {
        double sb = 0.0, sa = 0.0;
#pragma unroll
        for (int d = 0; d < IPF_MAXD; d++) {
            if (d < digits) {
                const double e = d == own_digit ? fp_from_u64(own_src[b * own_bs + (u64)x * n + jsrc])
                                                : ext[b * ext_bs + ((u64)d * ext_limbs + x) * n + jsrc];
                sb += fp_mulmod(e, kb[d], p, pinv);
                sa += fp_mulmod(e, ka[d], p, pinv);
            }
        }
        if (fold) sb = fp_norm(sb, p, pinv) + fp_mulmod(fp_from_u64(c0_src[b * own_bs + (u64)x * n + jsrc]), pm, p, pinv);
        u64* dst = acc + ((u64)s * n_batch + b) * acc_bs;
        dst[(u64)x * n + j] = fp_canonical(sb, p, pinv);
        dst[((u64)ext_limbs + x) * n + j] = fp_canonical(sa, p, pinv);
    }
}

// The sum over rotations, before the division by P: entry (s, b) of ext / own_src is term s of output b (its digits
// computed from the unrotated polynomial, gathered here through sigma_s like the own-digit limbs) -- or, with
// shared_input, entry b for every s: all terms of an output rotate the same ciphertext --
// acc[b] = sum_s sum_j sigma_s(e_{s,b,j}) * key_s[j].  A rotation's key values stay in registers across the IPS_BCH
// outputs of a block (4: many blocks for the few outputs of a layer; the blocks of a limb run together, so the key
// rows that each of them reads come from the L2 after the first); partial sums are normalised per rotation (eight terms of at most
// 0.875 * 2^50 stay below 2^53) and the running sums every eight rotations.
template <int IPS_BCH>
__global__ __launch_bounds__(IPF_NT) void inner_product_sum_fp_kernel(const FpPrime* fprimes, const double* ext, u64 ext_bs,
                                                                      int digits, int l, int K, int L, int alpha, IpSteps steps,
                                                                      int n_steps, int total, const u64* own_src, u64 own_bs,
                                                                      u64* acc, u64 acc_bs, u64 n_batch, int shared_input,
                                                                      int log_n) {
    const u64 n = (u64)1 << log_n;
    const uint32_t j = blockIdx.x * IPF_NT + threadIdx.x;
    const int x = blockIdx.z;      // the groups of outputs of a limb run together: they read the same key rows
    const u64 b0 = (u64)blockIdx.y * IPS_BCH;
    const int ext_limbs = l + K;
    const int prime = x < l ? x : L + (x - l);
    const int own_digit = x < l ? x / alpha : -1;
    const double p = as_const(&fprimes[prime].p)[0], pinv = as_const(&fprimes[prime].p)[1];
    double tb[IPS_BCH], ta[IPS_BCH];
#pragma unroll
    for (int u = 0; u < IPS_BCH; u++) tb[u] = ta[u] = 0.0;
    for (int s = 0; s < n_steps; s++) {
        const u64* key = steps.key[s];
        const uint32_t jsrc = galois_src_fp(j, steps.galois[s], log_n);
        double kb[IPF_MAXD], ka[IPF_MAXD];
#pragma unroll
        for (int d = 0; d < IPF_MAXD; d++) {
            if (d < digits) {
                kb[d] = fp_from_u64(key[(((u64)d * 2 + 0) * total + prime) * n + j]);
                ka[d] = fp_from_u64(key[(((u64)d * 2 + 1) * total + prime) * n + j]);
            }
        }
#pragma unroll
        for (int u = 0; u < IPS_BCH; u++) {
            if (b0 + u < n_batch) {
                const u64 entry = (shared_input ? 0 : (u64)s * n_batch) + b0 + u;
                double sb = 0.0, sa = 0.0;
#pragma unroll
                for (int d = 0; d < IPF_MAXD; d++) {
                    if (d < digits) {
                        const double e = d == own_digit ? fp_from_u64(own_src[entry * own_bs + (u64)x * n + jsrc])
                                                        : ext[entry * ext_bs + ((u64)d * ext_limbs + x) * n + jsrc];
                        sb += fp_mulmod(e, kb[d], p, pinv);
                        sa += fp_mulmod(e, ka[d], p, pinv);
                    }
                }
                tb[u] += fp_norm(sb, p, pinv);
                ta[u] += fp_norm(sa, p, pinv);
                if ((s & 7) == 7) { tb[u] = fp_norm(tb[u], p, pinv); ta[u] = fp_norm(ta[u], p, pinv); }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < IPS_BCH; u++) {
        if (b0 + u < n_batch) {
            u64* dst = acc + (b0 + u) * acc_bs;
            dst[(u64)x * n + j] = fp_canonical(tb[u], p, pinv);
            dst[((u64)ext_limbs + x) * n + j] = fp_canonical(ta[u], p, pinv);
        }
    }
}

hipError_t launch_inner_product_sum_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                       int alpha, const IpSteps& steps, int n_steps, int total, const u64* own_src, u64 own_bs,
                                       u64* acc, u64 acc_bs, u64 n_batch, int shared_input, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (digits < 1 || digits > IPF_MAXD || n_steps < 1 || n_steps > FP_MAX_STEPS || l < 1 || K < 1 || alpha < 1) return hipErrorInvalidValue;
    if (!fprimes || !ext || !own_src || !acc || n_batch == 0 || n_batch > 65535u * 4 || l + K > 65535) return hipErrorInvalidValue;
    // an entry holds `digits` extended digits of l + K limbs; an accumulator two polynomials of l + K limbs; an own-digit
    // source the l limbs of the polynomial
    const u64 n = (u64)1 << log_n;
    if (ext_bs < (u64)digits * (l + K) * n || acc_bs < (u64)2 * (l + K) * n || own_bs < (u64)l * n) return hipErrorInvalidValue;
    for (int s = 0; s < n_steps; s++)
        if (!steps.key[s] || steps.galois[s] == 0) return hipErrorInvalidValue;
    const unsigned bch = 4;
    dim3 grid((1u << log_n) / IPF_NT, (unsigned)((n_batch + bch - 1) / bch), l + K);
    ProfScope prof__("inner_product_sum_fp_kernel", st);
    hipLaunchKernelGGL(inner_product_sum_fp_kernel<4>, grid, dim3(IPF_NT), 0, st, fprimes, ext, ext_bs, digits, l, K, L, alpha,
                       steps, n_steps, total, own_src, own_bs, acc, acc_bs, n_batch, shared_input, log_n);
    return hipGetLastError();
}

hipError_t launch_inner_product_steps_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                         int alpha, const IpSteps& steps, int n_steps, int total, const u64* own_src,
                                         u64 own_bs, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st,
                                         const u64* c0_src, const u64* pmod) {
    DRY_RUN_RETURN();
    if (digits > IPF_MAXD || n_steps < 1 || n_steps > FP_MAX_STEPS) return hipErrorInvalidValue;
    if (!fprimes || !ext || !own_src || !acc || n_batch == 0 || (c0_src && !pmod)) return hipErrorInvalidValue;
    for (int s = 0; s < n_steps; s++)
        if (!steps.key[s] || steps.galois[s] == 0) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / IPF_NT, n_steps, l + K);
    ProfScope prof__("inner_product_steps_fp_kernel", st);
    hipLaunchKernelGGL(inner_product_steps_fp_kernel, grid, dim3(IPF_NT), 0, st, fprimes, ext, ext_bs, digits, l, K, L, alpha,
                       steps, total, own_src, own_bs, acc, acc_bs, n_batch, c0_src, pmod, log_n);
    return hipGetLastError();
}

hipError_t launch_inner_product_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                   int alpha, const u64* key, int total, const u64* own_src, u64 own_bs, u64 galois,
                                   int gather_ext, u64* acc, u64 acc_bs, u64 n_batch, int log_n, hipStream_t st) {
    DRY_RUN_RETURN();
    if (digits > IPF_MAXD) return hipErrorInvalidValue;  // the caller falls back to the integer path
    if (!fprimes || !ext || !key || !own_src || !acc) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / IPF_NT, IPF_ZSPLIT, l + K);
    ProfScope prof__("inner_product_fp_kernel", st);
    hipLaunchKernelGGL(inner_product_fp_kernel, grid, dim3(IPF_NT), 0, st, fprimes, ext, ext_bs, digits, l, K, L, alpha, key,
                       total, own_src, own_bs, galois, gather_ext, acc, acc_bs, n_batch, log_n);
    return hipGetLastError();
}

hipError_t launch_inner_product_fold_fp(const FpPrime* fprimes, const double* ext, u64 ext_bs, int digits, int l, int K, int L,
                                        int alpha, const u64* key, int total, const u64* own_src, u64 own_bs, u64 galois,
                                        int gather_ext, u64* acc, u64 acc_bs, u64 n_batch, int log_n, const IpFold& fold,
                                        hipStream_t st) {
    DRY_RUN_RETURN();
    if (digits < 1 || digits > IPF_MAXD || l < 1 || K < 1 || alpha < 1 || l + K > 65535) return hipErrorInvalidValue;
    if (!fprimes || !ext || !key || !own_src || !acc || !fold.pin_tab || !fold.post_p) return hipErrorInvalidValue;
    if (fold.add && (fold.add_polys < 1 || fold.add_polys > 2)) return hipErrorInvalidValue;
    const u64 n = (u64)1 << log_n;
    if (ext_bs < (u64)digits * (l + K) * n || acc_bs < (u64)2 * (l + K) * n || own_bs < (u64)l * n) return hipErrorInvalidValue;
    if (fold.add && (fold.add_bs < (u64)fold.add_polys * l * n || (fold.add_polys > 1 && fold.add_ps < (u64)l * n))) return hipErrorInvalidValue;
    dim3 grid((1u << log_n) / IPF_NT, IPF_ZSPLIT, l + K);
    ProfScope prof__("inner_product_fold_fp_kernel", st);
    hipLaunchKernelGGL(inner_product_fold_fp_kernel, grid, dim3(IPF_NT), 0, st, fprimes, ext, ext_bs, digits, l, K, L, alpha, key,
                       total, own_src, own_bs, galois, gather_ext, acc, acc_bs, n_batch, log_n, fold);
    return hipGetLastError();
}
