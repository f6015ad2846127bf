// Negacyclic NTT / inverse NTT over Z_q[X]/(X^N+1), N = 2^10 .. 2^16, batched
// over limb-polynomials.  Forward: natural order in, a(psi^(2*bitrev(i)+1)) at
// index i out (decimation in time, psi-twist merged into the twiddles).
// Inverse: the same levels undone in reverse order, then N^-1.
//
// A polynomial is processed in tiles of 2^11 coefficients staged in LDS
// (16 KiB, 256 threads).  Up to N = 2^11 one launch does all levels; above
// that a first launch does the top log2(N)-11 levels on tiles of
// 2^(log2 N - 11) rows x columns (rows 2^11 apart, columns contiguous, so
// global accesses stay coalesced) and a second launch does the remaining 11
// levels on contiguous tiles.  Butterflies are Harvey-style lazy (values below
// 4q forward, 2q inverse) with Shoup twiddles; only the last launch of a
// transform writes canonical residues.
#include "hisa_internal.hpp"
#include "modarith.hpp"

#define TILE_LOG 11
#define NT 256

struct PassArgs {
    u64* data;
    const u64* in;
    u64 batch_stride, in_batch_stride;
    int log_n;
    int s0, s1;        // this launch does levels s0+1 .. s1 (level s pairs elements N/2^s apart)
    int strided;       // 1: tile = rows 2^(log_n - s1) apart x contiguous columns; 0: contiguous tile
    int canonical_out; // 1: last launch of the transform
    u64 galois;        // inverse, first launch: gather through the NTT-form automorphism
    const u64* post;   // inverse, last launch: per-entry final factors (else N^-1)
    const u64* post_sh;
    int out_entry0;    // output polynomial of entry e sits at (e - out_entry0) * N within its batch slot
};

__device__ __forceinline__ uint32_t brev_bits(uint32_t x, int bits) { return __brev(x) >> (32 - bits); }

// index that the automorphism X -> X^g reads from, in NTT (bit-reversed evaluation) order
__device__ __forceinline__ uint32_t galois_src(uint32_t i, u64 g, int log_n) {
    uint32_t two_n_mask = (2u << log_n) - 1;
    uint32_t e = 2 * brev_bits(i, log_n) + 1;
    uint32_t e2 = (uint32_t)((u64)e * g) & two_n_mask;
    return brev_bits((e2 - 1) >> 1, log_n);
}

template <bool INV>
__global__ __launch_bounds__(NT) void ntt_pass_kernel(PassArgs a, NttTables t, PolyMap map) {
    __shared__ u64 lds[1 << TILE_LOG];
    const int tiles_log = a.log_n < TILE_LOG ? 0 : a.log_n - TILE_LOG;
    const int p = blockIdx.x >> tiles_log;
    const uint32_t tile = blockIdx.x & ((1u << tiles_log) - 1);
    const int entry = p % map.period;
    const int prime = map.prime_of[entry];
    if (prime < 0) return;
    const u64 n = (u64)1 << a.log_n;
    const int tile_log = a.log_n < TILE_LOG ? a.log_n : TILE_LOG;
    const int tile_elems = 1 << tile_log;
    const int levels = a.s1 - a.s0;
    const int logC = tile_log - levels; // columns per tile (strided) / sub-transforms per tile (contiguous)
    const u64 q = t.primes[prime].q;
    const u64 two_q = q << 1;
    const u64* tw = (INV ? t.itw : t.tw) + (u64)prime * n;
    const u64* tw_sh = (INV ? t.itw_sh : t.tw_sh) + (u64)prime * n;
    u64* base = a.data + (u64)(p / map.period) * a.batch_stride + (u64)(entry - a.out_entry0) * n;
    const u64* src = a.in ? a.in + (u64)(p / map.period) * a.in_batch_stride + (u64)entry * n : base;
    const u64 tile_base = a.strided ? ((u64)tile << logC) : ((u64)tile << tile_log);
    const int row_shift = a.log_n - a.s1; // log2 of the row distance of a strided tile

    // local index -> global coefficient index
    auto gidx = [&](int li) -> u64 {
        if (a.strided) return tile_base + ((u64)(li >> logC) << row_shift) + (li & ((1 << logC) - 1));
        return tile_base + li;
    };

    for (int li = threadIdx.x; li < tile_elems; li += NT) {
        u64 j = gidx(li);
        if (INV && a.galois) j = galois_src((uint32_t)j, a.galois, a.log_n);
        lds[li] = src[j];
    }
    __syncthreads();

    const int cfast_log = a.strided ? logC : 0;
    for (int step = 0; step < levels; step++) {
        const int lam = INV ? levels - step : step + 1; // local level
        const int s = a.s0 + lam;                        // global level
        const int dist_log = (levels - lam) + cfast_log;
        const int dist = 1 << dist_log;
        for (int x = threadIdx.x; x < tile_elems / 2; x += NT) {
            const int lo = x & (dist - 1);
            const int li = ((x >> dist_log) << (dist_log + 1)) | lo;
            const u64 j = gidx(li);
            const u64 widx = ((u64)1 << (s - 1)) + (j >> (a.log_n - s + 1));
            const u64 w = tw[widx], wp = tw_sh[widx];
            u64 X = lds[li], Y = lds[li + dist];
            if (!INV) {
                X = csub(X, two_q);
                u64 T = shoup_lazy(Y, w, wp, q);
                lds[li] = X + T;
                lds[li + dist] = X + two_q - T;
            } else {
                lds[li] = csub(X + Y, two_q);
                lds[li + dist] = shoup_lazy(X + two_q - Y, w, wp, q);
            }
        }
        __syncthreads();
    }

    u64 f = 0, f_sh = 0;
    if (INV && a.canonical_out) {
        if (a.post) { f = a.post[entry]; f_sh = a.post_sh[entry]; }
        else { f = t.primes[prime].n_inv; f_sh = t.primes[prime].n_inv_sh; }
    }
    for (int li = threadIdx.x; li < tile_elems; li += NT) {
        u64 v = lds[li];
        if (a.canonical_out) {
            if (INV) v = shoup_mul(v, f, f_sh, q);
            else v = csub(csub(v, two_q), q);
        }
        base[gidx(li)] = v;
    }
}

static hipError_t run_pass(bool inv, PassArgs a, const NttTables& t, const PolyMap& map, int n_polys, hipStream_t st) {
    int tile_log = a.log_n < TILE_LOG ? a.log_n : TILE_LOG;
    dim3 grid((unsigned)n_polys << (a.log_n - tile_log));
    ProfScope prof__(inv ? "ntt_pass_kernel<true>" : "ntt_pass_kernel<false>", st);
    if (inv) hipLaunchKernelGGL(ntt_pass_kernel<true>, grid, dim3(NT), 0, st, a, t, map);
    else hipLaunchKernelGGL(ntt_pass_kernel<false>, grid, dim3(NT), 0, st, a, t, map);
    return hipGetLastError();
}

// PolyMap -> compact task list of the fp64 single-launch transform; false when it does not fit
static bool fp_tasks(const NttTables& t, int log_n, const PolyMap& map, int n_polys, int out_entry0, FpTask* tk) {
    if (!t.fp_ok || log_n < 12 || log_n > 15 || n_polys % map.period != 0) return false;
    int cnt = 0;
    for (int e = 0; e < map.period; e++) {
        if (map.prime_of[e] < 0) continue;
        if (cnt >= HISA_MAX_PRIMES) return false;
        tk->pos[cnt] = (int16_t)(e - out_entry0);
        tk->prime[cnt] = map.prime_of[e];
        cnt++;
    }
    tk->period = cnt;
    return cnt > 0;
}

static FpArgs fp_base_args(const NttTables& t) {
    FpArgs a = {};
    a.fprimes = t.fprimes; a.ftw = t.ftw; a.utw = t.utw; a.vtw = t.vtw;
    return a;
}

hipError_t launch_ntt(const NttTables& t, int log_n, u64* data, u64 batch_stride, int n_polys, const PolyMap& map,
                      hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_polys <= 0) return hipSuccess;
    FpTask tk;
    if (fp_tasks(t, log_n, map, n_polys, 0, &tk)) {
        FpArgs fa = fp_base_args(t);
        fa.in = data; fa.in_bs = batch_stride; fa.out = data; fa.out_bs = batch_stride;
        return launch_ntt_fp(FP_FWD_PLAIN, log_n, fa, tk, (u64)(n_polys / map.period), st);
    }
    PassArgs a = {};
    a.data = data; a.in = nullptr; a.batch_stride = batch_stride; a.log_n = log_n;
    if (log_n <= TILE_LOG) {
        a.s0 = 0; a.s1 = log_n; a.strided = 0; a.canonical_out = 1;
        return run_pass(false, a, t, map, n_polys, st);
    }
    a.s0 = 0; a.s1 = log_n - TILE_LOG; a.strided = 1; a.canonical_out = 0;
    hipError_t e = run_pass(false, a, t, map, n_polys, st);
    if (e != hipSuccess) return e;
    a.s0 = log_n - TILE_LOG; a.s1 = log_n; a.strided = 0; a.canonical_out = 1;
    return run_pass(false, a, t, map, n_polys, st);
}

hipError_t launch_intt(const NttTables& t, int log_n, u64* data, u64 batch_stride, int n_polys, const PolyMap& map,
                       const InttExtra* extra, hipStream_t st) {
    DRY_RUN_RETURN();
    if (n_polys <= 0) return hipSuccess;
    FpTask tk;
    if ((!extra || !extra->post) && fp_tasks(t, log_n, map, n_polys, extra ? extra->out_entry0 : 0, &tk)) {
        FpArgs fa = fp_base_args(t);
        fa.in = (extra && extra->in) ? extra->in : data;
        fa.in_bs = (extra && extra->in) ? extra->in_batch_stride : batch_stride;
        fa.in_pos_shift = extra ? extra->out_entry0 : 0;
        fa.galois = extra ? extra->galois : 0;
        fa.out = data; fa.out_bs = batch_stride;
        return launch_ntt_fp(FP_INV_PLAIN, log_n, fa, tk, (u64)(n_polys / map.period), st);
    }
    PassArgs a = {};
    a.data = data; a.batch_stride = batch_stride; a.log_n = log_n;
    if (extra) {
        a.in = extra->in; a.in_batch_stride = extra->in_batch_stride; a.galois = extra->galois;
        a.out_entry0 = extra->out_entry0;
    }
    if (log_n <= TILE_LOG) {
        a.s0 = 0; a.s1 = log_n; a.strided = 0; a.canonical_out = 1;
        if (extra) { a.post = extra->post; a.post_sh = extra->post_sh; }
        return run_pass(true, a, t, map, n_polys, st);
    }
    a.s0 = log_n - TILE_LOG; a.s1 = log_n; a.strided = 0; a.canonical_out = 0;
    hipError_t e = run_pass(true, a, t, map, n_polys, st);
    if (e != hipSuccess) return e;
    a.in = nullptr; a.galois = 0;
    a.s0 = 0; a.s1 = log_n - TILE_LOG; a.strided = 1; a.canonical_out = 1;
    if (extra) { a.post = extra->post; a.post_sh = extra->post_sh; }
    return run_pass(true, a, t, map, n_polys, st);
}
