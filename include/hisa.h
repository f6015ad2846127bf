/*
 * hisa.h -- C ABI of libhisa: the HISA instruction set of the CHET paper
 * (Sec. "HISA", Fig. "Instructions of the HISA") over RNS-CKKS, executed by
 * hand-written HIP kernels on one AMD gfx950 GPU, plus the HW-tiled tensor
 * kernels of the paper's runtime (Sec. "Runtime", Algorithm 1).
 *
 * Conventions
 *  - Every function returns an int: HISA_OK (0) or a negative HISA_ERR_* code;
 *    hisa_last_error(ctx) gives a message owned by the context.  Nothing
 *    throws across this boundary.
 *  - hisa_ct / hisa_pt are opaque handles that own DEVICE memory.  The caller
 *    owns every handle it receives through an out-pointer and releases it
 *    with hisa_free (the table's `free`).  `*_assign` forms mutate their first
 *    argument in place (the table's `...Assign` instructions).
 *  - Pointers named host_* / plain `const double*`, `const int32_t*`,
 *    `uint64_t* host` are HOST pointers; `dev_*` are DEVICE pointers.
 *  - All work is enqueued on the HIP stream given to hisa_create (NULL = the
 *    default stream); functions that return data to the host synchronise that
 *    stream before returning.  A context is not thread-safe.
 *  - Ciphertexts are (c0, c1[, c2]) with c0 + c1*s (+ c2*s^2) ~ scale * message,
 *    kept in NTT form on the device, layout [poly][limb][N] of uint64 residues
 *    in [0, q_i); export/import use COEFFICIENT form with canonical residues,
 *    which is the representation the bit-exact parity tests compare.
 *  - Keys never cross the boundary in normal use (Sec. "HISA": key handling is
 *    the library's business); hisa_key_export exists for parity tests only.
 *  - No function falls back to the CPU: without a usable GPU hisa_create fails.
 */
#ifndef HISA_H
#define HISA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HISA_OK 0
#define HISA_ERR_ARG (-1)             /* null pointer, bad size, bad parameter          */
#define HISA_ERR_LEVEL_MISMATCH (-2)  /* operands carry different numbers of limbs      */
#define HISA_ERR_SCALE_MISMATCH (-3)  /* add/sub operands differ in scale (rel. 2^-30)   */
#define HISA_ERR_NO_KEY (-4)          /* rotation amount / relin without a generated key */
#define HISA_ERR_BAD_DIVISOR (-5)     /* divScalar with x != maxScalarDiv(c, ub)         */
#define HISA_ERR_DEPTH_EXHAUSTED (-6) /* rescale of a one-limb ciphertext                */
#define HISA_ERR_OOM (-7)             /* device allocation failed                        */
#define HISA_ERR_HIP (-8)             /* a HIP runtime call or kernel launch failed      */
#define HISA_ERR_SIZE (-9)            /* wrong number of polynomials for this operation  */

#define HISA_MAX_Q 48       /* most ciphertext primes                */
#define HISA_MAX_PRIMES 64  /* most ciphertext + special primes       */

typedef struct hisa_ctx hisa_ctx;
typedef struct hisa_ct hisa_ct;
typedef struct hisa_pt hisa_pt;

/*
 * Initialisation lies outside the HISA (Sec. "HISA", last paragraphs): ring
 * degree N = 2^log_n (N/2 complex slots), the ciphertext primes q_0..q_{L-1}
 * (q_bits[i] bits each, = 1 mod 2N, the largest unused such prime below
 * 2^bits), dnum key-switching digits of alpha = ceil(L/dnum) primes, alpha
 * special primes of special_bits bits, and the seed of all randomness.
 * noise = 1: discrete Gaussian errors; noise = 0: all error
 * polynomials zero (for exactness tests only).  Bits must lie in [log_n+2, 60].
 * sigma: parameter of the error distribution, pmf proportional to
 * exp(-x^2 / (2 sigma^2)) on |x| <= floor(6 sigma); 0 selects 3.2, otherwise
 * 0.2 < sigma <= 10.  secret_kind = 0: every secret coefficient uniform in
 * {-1, 0, 1}; 1: exactly hamming_weight non-zero coefficients (+-1) at
 * uniformly drawn positions (the sparse secrets of HEAAN),
 * 1 <= hamming_weight <= N.  Anything else is HISA_ERR_ARG.
 */
typedef struct {
    uint32_t log_n;               /* 10 .. 16 */
    uint32_t num_q;               /* L, 1 .. HISA_MAX_Q */
    uint32_t q_bits[HISA_MAX_Q];
    uint32_t dnum;                /* 1 .. L */
    uint32_t special_bits;
    uint32_t noise;
    uint64_t seed;
    double sigma;                 /* 0: 3.2 */
    uint32_t secret_kind;         /* 0 uniform ternary, 1 fixed Hamming weight */
    uint32_t hamming_weight;      /* secret_kind = 1 only */
} hisa_params;

/* hip_stream: a hipStream_t (may be NULL).  The context allocates its tables,
 * the ternary secret and a device memory pool; hisa_destroy releases all of it
 * (handles still alive become dangling). */
int hisa_create(const hisa_params* params, void* hip_stream, hisa_ctx** out);
int hisa_destroy(hisa_ctx* ctx);
const char* hisa_last_error(const hisa_ctx* ctx);
int hisa_sync(hisa_ctx* ctx);

/* Evaluation keys (Sec. "HEAAN": re-linearisation and rotation need keys).
 * hisa_keygen makes the re-linearisation key.  hisa_gen_rot_keys makes one key
 * per distinct left-rotation amount in host array left_steps[n] -- the paper's
 * rotation-key selection (Sec. "Rotation Keys Selection"); amounts are taken
 * modulo N/2, zero and repeats are skipped. */
int hisa_keygen(hisa_ctx* ctx);
int hisa_gen_rot_keys(hisa_ctx* ctx, const int32_t* left_steps, size_t n);

/* ---- Integers profile: encode / decode (Fig. "Instructions of the HISA") ----
 * The HEAAN family packs N/2 complex numbers (Sec. "HEAAN"); host arrays
 * re[count], im[count] (im may be NULL = real input), count <= N/2, missing
 * slots are zero.  The plaintext gets `limbs` limbs (1..L) and the given scale.
 * Slot j is the value at the root exp(i*pi*5^j/N), which makes rotLeft a cyclic
 * left shift.  Arithmetic is fp64, so encode is approximate (rounding error
 * O(sqrt N) per Sec. "HEAAN"), not bit-reproducible across implementations. */
int hisa_encode(hisa_ctx* ctx, const double* re, const double* im, size_t count, double scale, uint32_t limbs,
                hisa_pt** out);
int hisa_decode(hisa_ctx* ctx, const hisa_pt* pt, double* re, double* im, size_t count);
/* Exact route for parity tests: signed integer coefficients host_coeffs[N]. */
int hisa_pt_from_coeffs(hisa_ctx* ctx, const int64_t* host_coeffs, double scale, uint32_t limbs, hisa_pt** out);
/* host[limbs][N], coefficient form, canonical residues. */
int hisa_pt_export(hisa_ctx* ctx, const hisa_pt* pt, uint64_t* host);
int hisa_pt_info(const hisa_pt* pt, uint32_t* limbs, double* scale);

/* ---- Encryption profile ----
 * encrypt: symmetric, c1 = a uniform, c0 = -a*s + e + m, at the plaintext's
 * level; the context's encryption counter selects the random streams and is
 * advanced by one per ciphertext.  decrypt: c0 + c1*s (+ c2*s^2). */
int hisa_encrypt(hisa_ctx* ctx, const hisa_pt* pt, hisa_ct** out);
int hisa_decrypt(hisa_ctx* ctx, const hisa_ct* ct, hisa_pt** out);
int hisa_copy(hisa_ctx* ctx, const hisa_ct* ct, hisa_ct** out);
int hisa_free(hisa_ctx* ctx, void* handle); /* hisa_ct* or hisa_pt*; NULL is a no-op */
int hisa_set_enc_counter(hisa_ctx* ctx, uint64_t counter);

/* ---- add / sub: ciphertext, plaintext or scalar (limb-wise mod q_i) ----
 * Operands need equal limb counts and (for add/sub) equal scales.  The scalar
 * forms add round(x * scale) to the constant coefficient of c0, which shifts
 * every slot by x. */
int hisa_add(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out);
int hisa_sub(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out);
int hisa_add_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b);
int hisa_sub_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b);
int hisa_add_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out);
int hisa_sub_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out);
int hisa_add_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p);
int hisa_sub_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p);
int hisa_add_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, hisa_ct** out);
int hisa_sub_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, hisa_ct** out);
int hisa_add_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x);
int hisa_sub_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x);

/* ---- mul: ciphertext, plaintext or scalar; Relin profile ----
 * mul = mul_no_relin + relinearize.  mul_no_relin gives the three-polynomial
 * ciphertext (a0 b0, a0 b1 + a1 b0, a1 b1); relinearize (in place) brings it
 * back to two with the s^2 key.  mul_scalar multiplies every residue by the
 * integer round(x * x_scale) (the fixed-point conversion of a weight in
 * Algorithm 1, its precision the logarithm of x_scale); scales multiply. */
int hisa_mul(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out);
int hisa_mul_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_ct* b);
int hisa_mul_no_relin(hisa_ctx* ctx, const hisa_ct* a, const hisa_ct* b, hisa_ct** out);
int hisa_relinearize(hisa_ctx* ctx, hisa_ct* ct);
int hisa_mul_plain(hisa_ctx* ctx, const hisa_ct* a, const hisa_pt* p, hisa_ct** out);
int hisa_mul_plain_assign(hisa_ctx* ctx, hisa_ct* a, const hisa_pt* p);
int hisa_mul_scalar(hisa_ctx* ctx, const hisa_ct* a, double x, double x_scale, hisa_ct** out);
int hisa_mul_scalar_assign(hisa_ctx* ctx, hisa_ct* a, double x, double x_scale);

/* ---- rotations (the rotLeft / rotRight rows of Fig. "Instructions of the HISA") ----
 * rotLeft(r): (sigma_g(c0), 0) + KeySwitch_g(sigma_g(c1)), g = 5^r mod 2N;
 * rotRight(r) = rotLeft(N/2 - r); r = 0 (mod N/2) is a copy and needs no key;
 * any other amount needs its key from hisa_gen_rot_keys, else HISA_ERR_NO_KEY. */
int hisa_rot_left(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct** out);
int hisa_rot_right(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct** out);
int hisa_rot_left_assign(hisa_ctx* ctx, hisa_ct* a, int32_t steps);
int hisa_rot_right_assign(hisa_ctx* ctx, hisa_ct* a, int32_t steps);
/* rotLeft for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): out = rotLeft(a, steps), bit for bit what hisa_rot_left gives, written into the
 * EXISTING two-polynomial ciphertext `out` (same number of limbs as `a`, not overlapping it; its scale is set to
 * a's).  The call allocates nothing on the device: its intermediates (about (4 + ceil(l/alpha)) (l + K) + l
 * limb-polynomials of 8 N bytes) live in a static device array of HISA_NOALLOC_SCRATCH_BYTES inside the library, of
 * which every GPU the library runs on holds its own copy until the process ends.  A rotation that needs more returns
 * HISA_ERR_SIZE (the message names both sizes); N = 2^15 with 16 limbs and dnum 3 fits.  Needs what the fused key
 * switch needs (2^12 <= N <= 2^15, every prime below 2^50, dnum <= 8: HISA_ERR_ARG otherwise), the amount's key
 * (HISA_ERR_NO_KEY), per-kernel timing switched off, and the context's device current.  All calls on one GPU share
 * that GPU's array (contexts included), which keeps the last call's contents; every part is rewritten before it is
 * read, so nothing is cleared.  Calls that overlap in time on one GPU -- two contexts on different streams -- race on it:
 * the caller orders them. */
#define HISA_NOALLOC_SCRATCH_BYTES (36u << 20)
int hisa_rot_left_noalloc(hisa_ctx* ctx, const hisa_ct* a, int32_t steps, hisa_ct* out);

/* ---- Division profile, RNS reading (Sec. "HISA": the divisor is a coprime
 * modulus of the ciphertext) ----
 * max_scalar_div: the last modulus q_{l-1} of the ciphertext if l > 1 and it is
 * below ub, else 1.  div_scalar(d): d = 1 is a no-op; d must equal
 * max_scalar_div for some ub (else HISA_ERR_BAD_DIVISOR); rounds to nearest,
 * drops the last limb, divides the scale by d.  rescale = div_scalar by
 * max_scalar_div(ct, +inf). */
int hisa_max_scalar_div(hisa_ctx* ctx, const hisa_ct* ct, double ub, uint64_t* d);
int hisa_div_scalar(hisa_ctx* ctx, hisa_ct* ct, uint64_t d);
int hisa_rescale(hisa_ctx* ctx, hisa_ct* ct);

/* ---- batched forms: n ciphertexts of equal shape, one launch set ----
 * in[n] / out[n] are host arrays of handles; out receives n new handles that
 * are views of one device allocation.  rot_left_batch shares one rotation
 * amount (one key, read once per batch).  The *_assign_batch forms mutate. */
int hisa_rot_left_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n, int32_t steps, hisa_ct** out);
/* Several rotations of the same n ciphertexts: out[s*n + i] = rotLeft(in[i], steps[s]), bit for bit what
 * hisa_rot_left gives.  The digit decomposition and extension of c1 to the special primes (the first half of a key
 * switch) is computed once and shared by all steps: it works coefficient by coefficient on centred values, so it
 * commutes with the automorphism (the code motion of rotations of Sec. "Runtime", taken below the HISA boundary).
 * Needs every step's key (HISA_ERR_NO_KEY before any work is queued); on error no handle is returned. */
int hisa_rot_left_hoisted_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n, const int32_t* steps,
                                size_t n_steps, hisa_ct** out);
/* Sums of rotated ciphertexts: out[b] = sum over s of rotLeft(in[s*n_out + b], steps[s]), for n_out outputs of
 * n_terms terms each (the reduction over equally strided channels of Sec. "Homomorphic Tensor Operations", CHW
 * paragraph, when each channel's term is its own ciphertext).  The terms are decomposed and multiplied by their keys
 * one by one, but the accumulators on the l + K limbs are added up before the division by P, which is then taken once
 * per output: the result is the sum of the rotated ciphertexts up to the rounding of that division (ciphertext bits
 * differ from summing hisa_rot_left results).  When all rotated terms of every output are the same handle (a sum of
 * rotations of one ciphertext), that ciphertext is decomposed once (as in hisa_rot_left_hoisted_batch): same bits,
 * less work.  At most one step may be a multiple of the slot count (that term is
 * added as it is), at most 32 may rotate; all inputs share level and scale.  Needs N >= 2^12, every prime below 2^50
 * and dnum <= 8 (HISA_ERR_ARG otherwise), and every step's key (HISA_ERR_NO_KEY before any work is queued). */
int hisa_rot_left_sum_batch(hisa_ctx* ctx, const hisa_ct* const* in, size_t n_out, const int32_t* steps, size_t n_terms,
                            hisa_ct** out);
/* Rotate-and-add chains x += rot(x, s); x += rot(x, 2s); x += rot(x, 4s); .. (the log-step reductions and replications of
 * hisa_fc and hisa_matmul*) add up all multiples of s below 2^k s.  With max_doublings = 2..4 those layers take up to
 * that many consecutive doublings as ONE sum of the 2^c - 1 rotations by s, 2s, 3s, .. of the same ciphertext
 * (hisa_rot_left_sum_batch: one decomposition, one division by P) instead of c key switches one after the other:
 * more rotation keys (hisa_fc_rot_steps / hisa_matmul_rot_steps list them), fewer and larger launches; the same sums
 * up to the rounding of the divisions, other ciphertext bits.  hisa_sum_pool2x2 then takes its four corners as one
 * such sum as well.  0 (the default) keeps the chains.  Needs what
 * hisa_rot_left_sum_batch needs (HISA_ERR_ARG otherwise, and for other values).  A plan prepared under one setting
 * must be applied under the same one (the plaintexts do not depend on it, the rotation keys do). */
int hisa_set_merge_doublings(hisa_ctx* ctx, uint32_t max_doublings);
/* Where a layer's division by P (the end of its key switches) is directly followed by its divScalar by the last
 * modulus, on = 1 makes it take both at once: the accumulators on the l + K limbs (with the terms that were not
 * rotated folded in, times P) are divided by q_{l-1} P in one base conversion whose sources are the limb of q_{l-1} and
 * the special limbs.  One inverse and l - 1 forward transforms per polynomial instead of two rounds of them; the result
 * differs from the two-step one by the rounding of the conversion (a few units per coefficient), so ciphertext bits
 * differ.  Applies to the CHW-tiled convolutions that rotate sums, the shared_moddown convolution with scalar weights and the
 * degree-2 activation; 0 (the default) keeps the two steps.  Needs what
 * hisa_rot_left_sum_batch needs (HISA_ERR_ARG otherwise).  A setting of the context, like hisa_set_merge_doublings. */
int hisa_set_fused_rescale(hisa_ctx* ctx, uint32_t on);
int hisa_relinearize_batch(hisa_ctx* ctx, hisa_ct* const* cts, size_t n);
int hisa_rescale_batch(hisa_ctx* ctx, hisa_ct* const* cts, size_t n);
int hisa_add_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_ct* const* b, size_t n, hisa_ct** out);
int hisa_mul_plain_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_pt* p, size_t n, hisa_ct** out);
int hisa_mul_no_relin_batch(hisa_ctx* ctx, const hisa_ct* const* a, const hisa_ct* const* b, size_t n,
                            hisa_ct** out);
int hisa_encrypt_batch(hisa_ctx* ctx, const hisa_pt* const* pts, size_t n, hisa_ct** out);
/* n ciphertexts (2 polynomials, `limbs` limbs) whose residues are uniform
 * random words of stream `counter`: synthetic benchmark inputs that are
 * indistinguishable from encryptions. */
int hisa_ct_random_batch(hisa_ctx* ctx, size_t n, uint32_t limbs, double scale, uint64_t counter, hisa_ct** out);

/* ---- analysis backend (Sec. "Compiler": the analyser executes the circuit on a
 * HISA backend that records instead of computing; used for the rotation-key
 * selection, the depth a circuit needs and the operation counts of the layout
 * cost model) ----
 * Between hisa_analysis_begin and hisa_analysis_end every call on this context
 * is a dry run: no kernel is launched, handles are still allocated and carry
 * their level and scale as in a real run (their contents are undefined), a
 * rotation whose key is missing is recorded instead of failing, and the
 * relinearisation key is not needed.  hisa_analysis_end leaves the mode and
 * returns what was recorded: the operation counts (in ciphertext operations;
 * the terms of the layers' fused multiply-accumulate launches are counted apart
 * from stand-alone multiplications and their additions are not counted),
 * for every count the sum of the limbs its operations ran on and the sum of their squares (limb_sum, limb_sq_sum, in
 * the order of the counts: what a cost that is a polynomial of degree two in the level needs, Sec. "Data Layout
 * Selection"),
 * the lowest limb count any ciphertext reached, and the sorted left-rotation
 * amounts that needed a key (at most cap of them into host rot_steps, the count
 * into *n; rot_steps may be null).  Handles made during the analysis stay valid
 * handles and are freed as usual.  Keys and plans cannot be made in this mode
 * (hisa_keygen, hisa_gen_rot_keys, hisa_*_prepare: HISA_ERR_ARG -- they would
 * hold no data), and a convolution asked for shared_moddown is counted in its
 * term-by-term schedule.  Not re-entrant: begin while already in analysis mode,
 * or end outside it, is HISA_ERR_ARG.  One context per thread at a time may be
 * in analysis mode. */
typedef struct {
    uint64_t rot_left;     /* key-switched rotations (rotRight counts here too) */
    uint64_t rot_shared;   /* of those, rotations that reused another rotation's decomposition */
    uint64_t rot_summed;   /* of those, rotations inside a sum that takes its division by P once (hisa_rot_left_sum_batch) */
    uint64_t relinearize, mul, mul_plain, mul_scalar, add, rescale;
    uint64_t mac_plain;    /* terms x * plaintext summed inside the layers' fused multiply-accumulate launches */
    uint64_t mac_scalar;   /* terms x * scalar weight summed there */
    uint64_t key_switch_calls; /* batched launches behind rot_left and relinearize: one per (call, rotation amount);
                                  a small batch costs its launch latency, not its share of the throughput */
    uint32_t min_limbs;    /* 0 if no ciphertext was made */
    uint32_t reserved;
    uint64_t limb_sum[12]; /* per count above, in that order: sum over its occurrences of the limbs they ran on */
    uint64_t limb_sq_sum[12]; /* and of the squares of those limbs */
} hisa_op_counts;
enum { HISA_OP_ROT_LEFT = 0, HISA_OP_ROT_SHARED, HISA_OP_ROT_SUMMED, HISA_OP_RELINEARIZE, HISA_OP_MUL, HISA_OP_MUL_PLAIN,
       HISA_OP_MUL_SCALAR, HISA_OP_ADD, HISA_OP_RESCALE, HISA_OP_MAC_PLAIN, HISA_OP_MAC_SCALAR, HISA_OP_KEY_SWITCH_CALLS };
int hisa_analysis_begin(hisa_ctx* ctx);
int hisa_analysis_end(hisa_ctx* ctx, hisa_op_counts* counts, int32_t* rot_steps, size_t cap, size_t* n);

/* ---- tensor layer (Sec. "Runtime": CipherTensor, HW- and CHW-tiling, Algorithm 1) ----
 * A CipherTensor is a vector of ciphertexts plus plain-integer metadata.
 * HW-tiling (c_inner = 1): the outer (batch, channel) dimensions index
 * ciphertexts cts[b*channels + c]; one ciphertext holds the height x width
 * plane of one channel, element (y, x) in slot offset + y*h_stride + x*w_stride
 * (strides leave room for padding between rows).  CHW-tiling (c_inner > 1):
 * c_inner channels share a ciphertext, c_stride slots apart: channel c of image
 * b is in cts[b*ceil(channels/c_inner) + c/c_inner], element (y, x) in slot
 * offset + (c mod c_inner)*c_stride + y*h_stride + x*w_stride; a last
 * ciphertext with fewer channels leaves the rest of its slots unused.  `clean`
 * is the runtime's flag that every slot that holds no element is zero.  The
 * struct is host memory owned by the caller; the handles in cts are owned like
 * any other handle.  Layer calls fill *out: out->cts must point to room for the
 * output handles.  hisa_fc takes HW-tiled tensors (HISA_ERR_ARG otherwise);
 * conv2d, pool, activation, matmul, mask, encrypt and decrypt take both. */
typedef struct {
    uint32_t batch, channels;    /* logical outer dimensions                  */
    uint32_t height, width;      /* logical inner dimensions                  */
    uint32_t h_stride, w_stride; /* physical strides in slots                 */
    uint32_t offset;             /* slot of element (0,0) of the first channel of a ciphertext */
    uint32_t clean;              /* 1: slots outside the elements hold zeros  */
    uint32_t c_inner;            /* channels per ciphertext (0 is read as 1)  */
    uint32_t c_stride;           /* slots between channels of one ciphertext  */
    hisa_ct** cts;               /* batch*ceil(channels/c_inner) handles      */
} hisa_tensor;

#define HISA_CONV_SCALAR 0 /* literal Algorithm 1: mulScalar by round(w * q_last), add, one divScalar; the output */
                           /* is not clean, except for a 1x1 stride-1 filter on a clean input                   */
#define HISA_CONV_MASKED 1 /* weights at scale q_last / 2^25, then ONE mulPlain by the 0/1 mask of the valid    */
                           /* output positions (scale 2^25) before the divScalar: the output is clean          */
#define HISA_PAD_SAME 1
#define HISA_PAD_SAME_MASKED 2
#define HISA_CONV_PLAIN 2  /* one mulPlain per tap: plaintext = w * mask encoded at scale q_last                 */
#define HISA_MASK_SCALE 33554432.0 /* 2^25 */

typedef struct {
    uint32_t fh, fw;      /* filter height, width                                                      */
    uint32_t stride;      /* output stride (>= 1)                                                      */
    uint32_t pad_same;    /* 0: VALID.  1 (HISA_PAD_SAME): SAME -- the input tensor must be clean and   */
                          /* its layout must leave fh/2 rows and fw/2 columns of zero slots around the */
                          /* plane.  2 (HISA_PAD_SAME_MASKED): SAME with the padding carried by the     */
                          /* weights: CHW-tiled tensors only (HISA_ERR_ARG otherwise, and with          */
                          /* shared_moddown); the plaintext of a tap is zero on the outputs whose input */
                          /* element under that tap lies outside the plane, so the layout needs no      */
                          /* border (planes can be packed back to back) and whatever a rotation brings  */
                          /* in from the neighbouring row, plane or block is multiplied by zero         */
    uint32_t mode;        /* HISA_CONV_*                                                              */
    uint32_t shared_moddown; /* 1: one division by P per output ciphertext instead of one per rotation: the   */
                          /* rotated taps enter the sum as their key-switch accumulators on the l + K limbs   */
                          /* (weights taken on those limbs), ModDown once at the end.  Same values up to the  */
                          /* rounding of that division; ciphertext bits differ from the schedule with         */
                          /* shared_moddown = 0.  Needs N >= 2^12, every prime below 2^50, dnum <= 8           */
                          /* (HISA_ERR_ARG otherwise); hisa_conv2d_fixed takes the same arguments              */
    uint32_t chw_schedule; /* CHW-tiled inputs only (ignored when c_inner = 1): HISA_CHW_*                    */
} hisa_conv_geom;
#define HISA_CHW_ROTATE_INPUTS 0 /* every input ciphertext is rotated by (tap, d); the products are summed         */
#define HISA_CHW_ROTATE_SUMS 1   /* the reduction over the channels of a ciphertext comes after the multiplication  */
                                 /* (Sec. "Homomorphic Tensor Operations", CHW paragraph): inputs are rotated by   */
                                 /* the taps only; for each output ciphertext and diagonal d the products are      */
                                 /* summed where the input channels lie (the plaintext of (tap, d, j, g) holds the */
                                 /* weight for output block b on block b + d; behind the blocks lies their copy,   */
                                 /* or block 0 when they fill the slots) and the c_inner sums are rotated left by  */
                                 /* d*c_stride and added by hisa_rot_left_sum_batch's arithmetic: one division by  */
                                 /* P per output ciphertext.  (taps - 1) rotations per input ciphertext plus       */
                                 /* c_inner - 1 key switches per output ciphertext instead of taps*c_inner - 1 per */
                                 /* input ciphertext; the same multiplications.  Needs what that call needs and    */
                                 /* c_inner <= 33; not together with shared_moddown (HISA_ERR_ARG).                */
#define HISA_CHW_ROTATE_SUMS_TAPS 2 /* the same with the two factors of the rotations exchanged: inputs are rotated  */
                                 /* by the d blocks only (d = 0..c_inner-1); for each output ciphertext and filter   */
                                 /* tap the products are summed under the input elements (the plaintext holds the    */
                                 /* weight of output position p on slot p + tap amount) and the per-tap sums are     */
                                 /* rotated by the taps and added, one division by P per output ciphertext.          */
                                 /* (c_inner - 1) rotations per input ciphertext plus taps - 1 key switches per      */
                                 /* output ciphertext; at most 33 taps, exactly one of them without a rotation.      */

/* HW-tiled conv2d (Algorithm 1; cross-correlation, no kernel flip): for every
 * output channel oc: sum over ic and filter taps (fy, fx) of weight *
 * rotLeft(in[ic], fy*h_stride + fx*w_stride) (SAME: taps are centred, negative
 * amounts rotate right), then one divScalar by the last modulus.  Rotations are
 * computed once per (ic, tap), batched over ic, and shared by all oc.  host
 * weights w[FH][FW][IC][OC].  Output strides are the input strides times the
 * conv stride.  Needs the rotation keys listed by hisa_conv2d_rot_steps.
 * hisa_conv2d_fixed takes the fixed-point integers directly (what
 * FixedPrecision(weight, plainLogP) and the plaintext encodings produce), so
 * that two implementations can be fed identical integers:
 *   SCALAR / MASKED: w_int[FH][FW][IC][OC] (scale w_scale); MASKED also
 *   pt_coeffs[N], the mask plaintext's signed coefficients (scale pt_scale);
 *   PLAIN: pt_coeffs[FH][FW][IC][OC][N] (scale pt_scale), w_int unused.
 * w_scale * pt_scale (or pt_scale alone for PLAIN, w_scale for SCALAR) should
 * equal the last modulus for the ciphertext scale to be preserved. */
/* CHW-tiled input (c_inner > 1; Sec. "Homomorphic Tensor Operations", CHW
 * paragraph: different weights on the channels of one ciphertext need mulPlain,
 * and the channels of a ciphertext are combined with rotations by the channel
 * stride): the mode must be HISA_CONV_PLAIN and the input clean (HISA_ERR_ARG
 * otherwise; hisa_tensor_mask cleans a tensor).  The c_inner channel blocks are
 * combined along diagonals: for d = 0..c_inner-1 output block b reads input
 * block (b+d) mod c_inner, so every input ciphertext is rotated once per
 * (tap, d), by tap amount + d*c_stride, and output ciphertext g is
 *   divScalar( sum over taps, d, input ciphertexts j of
 *              mulPlain(rot(x_j, tap, d), P[tap][d][j][g]) ),
 * P holding on the valid output positions of block b the weight from input
 * channel j*c_inner + (b+d) mod c_inner to output channel g*c_inner + b (zero
 * where either does not exist), at scale q_last.  The block rotation is cyclic
 * only if c_inner*c_stride equals the slot count; otherwise the blocks are first
 * copied once behind themselves (x += rotRight(x, c_inner*c_stride); needs
 * 2*c_inner*c_stride <= slots, else HISA_ERR_ARG).  fh*fw*c_inner is at most 256.
 * Output: clean, CHW-tiled with the same c_inner and c_stride,
 * batch*ceil(out_channels/c_inner) handles.  hisa_conv2d_fixed then takes
 * pt_coeffs[FH][FW][c_inner][ceil(IC/c_inner)][ceil(OC/c_inner)][N] (for either
 * chw_schedule; the plaintexts differ in where their blocks lie). */
int hisa_conv2d(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t out_channels,
                const hisa_conv_geom* geom, hisa_tensor* out);
int hisa_conv2d_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* w_int, double w_scale,
                      const int64_t* pt_coeffs, double pt_scale, uint32_t out_channels, const hisa_conv_geom* geom,
                      hisa_tensor* out);
/* The same convolution with its weights converted ahead of time (fixed-point residues per limb, the forms the
 * multiply-accumulate kernels read, the mask or per-tap plaintexts): hisa_conv2d_prepare builds a plan for tensors
 * with the layout, clean flag and level of `like`; hisa_conv2d_apply(in, plan) returns bit for bit what
 * hisa_conv2d(in, w, ...) returns.  Another layout is HISA_ERR_ARG, another level HISA_ERR_LEVEL_MISMATCH.  The plan
 * owns device memory until hisa_conv_plan_free. */
typedef struct hisa_conv_plan hisa_conv_plan;
int hisa_conv2d_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t out_channels,
                        const hisa_conv_geom* geom, hisa_conv_plan** plan);
int hisa_conv2d_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_plan* plan, hisa_tensor* out);
/* Several convolutions of the same tensor (the two expansion branches of a fire module of the SqueezeNet-style network
 * of Sec. "Evaluation"; the reuse of a rotated ciphertext in Algorithm 1, taken across layers):
 * outs[k] = hisa_conv2d_apply(in, plans[k]) bit for bit, but the plans that rotate their inputs (CHW_ROTATE_INPUTS by
 * (tap, diagonal), CHW_ROTATE_SUMS by the taps, CHW_ROTATE_SUMS_TAPS by the diagonals, HW-tiled by the taps; not those
 * with shared_moddown) take them from one set of hoisted rotations by the union of their amounts: an amount that two
 * plans ask for is rotated once.  plans and outs are host arrays of n_plans pointers; every outs[k] is prepared by the
 * caller like the output of hisa_conv2d_apply.  On an error no output is left allocated. */
int hisa_conv2d_apply_multi(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_plan* const* plans, size_t n_plans,
                            hisa_tensor* const* outs);
int hisa_conv_plan_free(hisa_ctx* ctx, hisa_conv_plan* plan);
/* Fully connected layer over all elements of all channels (Sec. "Homomorphic
 * matmul", the version without replicas): host w[OUT][C][H][W]; per output o:
 * sum_c mulPlain(in[c], encode(w[o][c] placed on the element slots, zero
 * elsewhere, scale q_last)), one divScalar, then a log-step rotate-and-add
 * (Sec. "Homomorphic Tensor Operations": reductions over equally strided
 * elements): amounts w_stride*2^k then h_stride*2^k with each dimension
 * rounded up to a power of two (the extra positions are zero after the masked
 * multiply) when the padded rows do not overlap and the padded plane stays
 * inside the slot vector, else -- or when that is not shorter -- 1, 2, 4, ..
 * over the contiguous window that covers the plane; hisa_fc_rot_steps lists
 * them.  Output o is a 1x1 plane in
 * slot `offset` (other slots hold partial sums: clean = 0).  On a 1x1 input it
 * is Algorithm 1 with a 1x1 filter (mulScalar, no rotations).
 * hisa_fc_fixed: pt_coeffs[OUT][C][N] signed plaintext coefficients at pt_scale. */
int hisa_fc(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t out_features, hisa_tensor* out);
int hisa_fc_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* pt_coeffs, double pt_scale,
                  uint32_t out_features, hisa_tensor* out);
/* The same layer with its weights encoded ahead of time (they are constants of the circuit; Sec. "Runtime" keeps
 * PlainTensors beside CipherTensors).  hisa_fc_prepare encodes w[OUT][C][H][W] for tensors with the layout and level
 * of `like` (only its metadata and its ciphertexts' limb count are read) into a plan that owns OUT*C plaintexts in
 * device memory (OUT*C*limbs*N*8 bytes) until hisa_fc_plan_free.  hisa_fc_apply(in, plan) returns bit for bit what
 * hisa_fc(in, w) returns; a tensor with another layout is HISA_ERR_ARG, another level HISA_ERR_LEVEL_MISMATCH.
 * Not for 1x1 planes (those multiply by scalars: HISA_ERR_ARG). */
typedef struct hisa_fc_plan hisa_fc_plan;
int hisa_fc_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t out_features, hisa_fc_plan** plan);
int hisa_fc_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_fc_plan* plan, hisa_tensor* out);
int hisa_fc_plan_free(hisa_ctx* ctx, hisa_fc_plan* plan);
/* The masking multiply as a layer (Sec. "Homomorphic Tensor Operations", SAME
 * padding: invalid elements are masked out with one mulPlain): every ciphertext
 * times the 0/1 vector of its element slots, encoded at the scale of the last
 * modulus, then divScalar: same values and scale, one level lower, clean = 1.
 * hisa_tensor_mask_fixed takes mask_coeffs[ceil(C/c_inner)][N] at mask_scale. */
int hisa_tensor_mask(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out);
/* A bias per channel after a linear layer (Algorithm 1 has none; Fig. "Instructions of the HISA" offers addPlain for
 * it).  In place: every ciphertext of t gets, by one addPlain, the vector that holds bias[c] (host, t->channels
 * values) on the element slots of each channel c it carries and zero elsewhere, encoded at the ciphertexts' own
 * scale -- level, scale and `clean` stay as they are.  All ciphertexts of t must be at one scale
 * (HISA_ERR_SCALE_MISMATCH); |bias[c]| * scale must stay below 2^62 (HISA_ERR_ARG: rescale first).
 * hisa_tensor_add_bias_fixed takes the encoded integers bias_coeffs[ceil(C/c_inner)][N] instead. */
int hisa_tensor_add_bias(hisa_ctx* ctx, hisa_tensor* t, const double* bias);
int hisa_tensor_add_bias_fixed(hisa_ctx* ctx, hisa_tensor* t, const int64_t* bias_coeffs);
int hisa_tensor_mask_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* mask_coeffs, double mask_scale,
                           hisa_tensor* out);
/* Layout switches (Sec. "Data Layout Selection": the layouts that change the
 * tiling around a layer).
 * hisa_tensor_to_chw: clean HW-tiled tensor -> CHW-tiled with c_inner channels
 * per ciphertext, c_stride slots apart: channel g*c_inner + k is rotated right
 * by k*c_stride and the channels of a group are added; no level is used; a
 * tensor that is not clean, or blocks that do not fit the slots: HISA_ERR_ARG.
 * hisa_tensor_to_hw: CHW-tiled tensor -> clean HW-tiled tensor: every
 * ciphertext is rotated left by k*c_stride for its blocks k (one shared
 * decomposition), each result times the 0/1 vector of the plane's slots
 * (scale of the last modulus), divScalar: one level.  The _fixed form takes the
 * mask as mask_coeffs[N] at mask_scale.  hisa_tensor_layout_rot_steps lists the
 * rotation amounts: of to_hw if `in` is CHW-tiled (c_inner, c_stride ignored),
 * else of to_chw(c_inner, c_stride). */
int hisa_tensor_to_chw(hisa_ctx* ctx, const hisa_tensor* in, uint32_t c_inner, uint32_t c_stride, hisa_tensor* out);
int hisa_tensor_to_hw(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out);
int hisa_tensor_to_hw_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* mask_coeffs, double mask_scale,
                            hisa_tensor* out);
int hisa_tensor_layout_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, uint32_t c_inner, uint32_t c_stride, int32_t* steps,
                                 size_t cap, size_t* n);
/* Homomorphic matmul with replicas (Sec. "Homomorphic Tensor Operations",
 * paragraphs "Homomorphic matmul" and "CHW-tiled convolution": replicas cost
 * log-many rotations and divide the number of mulPlain; reductions over equally
 * strided elements take log-many rotations).  Input: any tensor, HW- or
 * CHW-tiled; host w[OUT][C][H][W].  With P the power of two that covers the
 * element slots of a ciphertext and R the largest power of two that is at most
 * `replicas` and at most slots/P:
 *   1. (R > 1, input not clean) mulPlain by the 0/1 mask of the element slots,
 *      encoded at the scale of the last modulus, and divScalar: one level;
 *   2. (R > 1) log2 R times x += rotRight(x, P*2^k): R copies, P slots apart;
 *   3. per group g of R outputs: sum over the input ciphertexts of
 *      mulPlain(x_j, plaintext holding the weights of output gR+r on copy r),
 *      one divScalar;
 *   4. rotate-and-add inside the blocks (amounts as in hisa_fc, with the channel
 *      stride as a third strided dimension and the padded elements confined to
 *      the block when R > 1).
 * Output: OUT channels of 1x1 planes, CHW-tiled: c_inner = R, c_stride = P,
 * output gR+r in slot r*P + offset of ciphertext g; batch*ceil(OUT/R) handles
 * (hisa_matmul_geometry gives P, R and that count), clean = 0.  With R = 1 on an
 * HW-tiled input this is hisa_fc bit for bit.  Needs the rotation keys listed
 * by hisa_matmul_rot_steps, and two levels (one when R = 1 or the input is
 * clean): HISA_ERR_DEPTH_EXHAUSTED otherwise.
 * hisa_matmul_fixed takes the fixed-point plaintexts directly:
 * pt_coeffs[ceil(OUT/R)][ceil(C/c_inner)][N] signed coefficients at pt_scale and
 * (when step 1 applies, else null) mask_coeffs[ceil(C/c_inner)][N] at mask_scale.
 * hisa_matmul_prepare encodes the weights once for tensors with the layout,
 * clean flag and level of `like` into a plan that owns device memory until
 * hisa_matmul_plan_free; hisa_matmul_apply(in, plan) returns bit for bit what
 * hisa_matmul(in, w, ...) returns (another layout: HISA_ERR_ARG, another level:
 * HISA_ERR_LEVEL_MISMATCH). */
typedef struct hisa_matmul_plan hisa_matmul_plan;
int hisa_matmul_geometry(hisa_ctx* ctx, const hisa_tensor* in, uint32_t out_features, uint32_t replicas,
                         uint32_t* block, uint32_t* used_replicas, uint32_t* out_cts);
int hisa_matmul_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, uint32_t replicas, int32_t* steps, size_t cap, size_t* n);
int hisa_matmul(hisa_ctx* ctx, const hisa_tensor* in, const double* w, uint32_t out_features, uint32_t replicas,
                hisa_tensor* out);
int hisa_matmul_fixed(hisa_ctx* ctx, const hisa_tensor* in, const int64_t* pt_coeffs, double pt_scale,
                      const int64_t* mask_coeffs, double mask_scale, uint32_t out_features, uint32_t replicas,
                      hisa_tensor* out);
int hisa_matmul_prepare(hisa_ctx* ctx, const hisa_tensor* like, const double* w, uint32_t out_features, uint32_t replicas,
                        hisa_matmul_plan** plan);
int hisa_matmul_apply(hisa_ctx* ctx, const hisa_tensor* in, const hisa_matmul_plan* plan, hisa_tensor* out);
int hisa_matmul_plan_free(hisa_ctx* ctx, hisa_matmul_plan* plan);
/* 2x2 sum pool, stride 2 (the 1/4 of the average belongs in the next layer's
 * weights): x + rot(w_stride) + rot(h_stride) + rot(h_stride + w_stride);
 * strides double, no level is used. */
int hisa_sum_pool2x2(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out);
/* 2x2 average pool, stride 2: hisa_sum_pool2x2 whose outputs carry four times the scale.  A ciphertext stands for
 * (integer polynomial) / scale, so the larger scale is the division by 4: exact, no ciphertext operation, no level.
 * Layers after it see ciphertexts at that scale (a rescale divides it by the last modulus as usual). */
int hisa_avg_pool2x2(hisa_ctx* ctx, const hisa_tensor* in, hisa_tensor* out);
/* Degree-2 activation a*x^2 + b*x computed as x^2 + (b/a)*x: one mul with
 * relinearisation, one mulScalar by b/a at scale = ciphertext scale, one add,
 * one divScalar.  The factor a belongs in the next layer's weights. */
int hisa_poly2_act(hisa_ctx* ctx, const hisa_tensor* in, double a, double b, hisa_tensor* out);
/* The left-rotation amounts a layer will use on this input layout, for
 * hisa_gen_rot_keys (the rotation-key selection of Sec. "Rotation Keys
 * Selection"): writes at most cap amounts to host steps[], the count to *n.
 * For a convolution they depend on geom->chw_schedule as well as on the filter. */
int hisa_conv2d_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, const hisa_conv_geom* geom, int32_t* steps, size_t cap,
                          size_t* n);
int hisa_fc_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, int32_t* steps, size_t cap, size_t* n);
int hisa_pool_rot_steps(hisa_ctx* ctx, const hisa_tensor* in, int32_t* steps, size_t cap, size_t* n);
/* Encrypts a plain tensor host x[batch][channels][height][width] into a clean
 * CipherTensor with the tiling (c_inner, c_stride), strides and offset that
 * *inout names, at `limbs` limbs; elements that would share a slot are
 * HISA_ERR_ARG. */
int hisa_tensor_encrypt(hisa_ctx* ctx, const double* x, double scale, uint32_t limbs, hisa_tensor* inout);
/* Decrypts and decodes the elements back: host x[batch][channels][height][width]. */
int hisa_tensor_decrypt(hisa_ctx* ctx, const hisa_tensor* t, double* x);
int hisa_tensor_free(hisa_ctx* ctx, hisa_tensor* t);

/* ---- parity / debug surface ----
 * get_primes: host q[L], p[alpha].  ct_export: host[polys][limbs][N],
 * COEFFICIENT form, canonical residues.  ct_import: the inverse (new handle).
 * ntt_raw: in-place forward (inverse != 0: inverse) negacyclic NTT of n_polys
 * consecutive device polynomials dev_buf[n_polys][N] modulo prime prime_index
 * (0..L-1: q_i, L..L+alpha-1: special); forward output index i holds
 * a(psi^(2*bitrev(i)+1)).  key_export: host[dnum][2][L+alpha][N], NTT form,
 * (b, a) per digit; key_id 0 = relinearisation key, else a Galois element. */
int hisa_get_primes(hisa_ctx* ctx, uint64_t* q, uint64_t* p);
int hisa_get_alpha(hisa_ctx* ctx, uint32_t* alpha);
int hisa_ct_info(const hisa_ct* ct, uint32_t* limbs, uint32_t* polys, double* scale);
int hisa_ct_export(hisa_ctx* ctx, const hisa_ct* ct, uint64_t* host);
int hisa_ct_import(hisa_ctx* ctx, const uint64_t* host, uint32_t polys, uint32_t limbs, double scale, hisa_ct** out);
int hisa_ct_import_batch(hisa_ctx* ctx, const uint64_t* host, size_t n, uint32_t polys, uint32_t limbs, double scale,
                         hisa_ct** out);
int hisa_ct_device_ptr(const hisa_ct* ct, uint64_t** dev);
int hisa_ntt_raw(hisa_ctx* ctx, uint64_t* dev_buf, uint32_t prime_index, size_t n_polys, int inverse);
int hisa_key_export(hisa_ctx* ctx, uint64_t key_id, uint64_t* host);
int hisa_galois_elt(hisa_ctx* ctx, int32_t left_steps, uint64_t* g);
int hisa_secret_export(hisa_ctx* ctx, int64_t* host_coeffs);


/* ---- measurement ----
 * profile_enable(1) brackets every kernel launch of the process with HIP events
 * recorded on the context's stream; profile_read synchronises, writes one line
 * per kernel name ("name<TAB>launches<TAB>total milliseconds") into host_buf
 * (cap bytes, NUL-terminated) and clears the records.  Off by default; meant for
 * a separate measuring pass, not for timed runs. */
int hisa_profile_enable(hisa_ctx* ctx, int on);
int hisa_profile_read(hisa_ctx* ctx, char* host_buf, size_t cap);

/* ---- measurement support (not a HISA instruction) ----
 * Peaks of the GPU the context lives on, measured: issue rates, in 10^12 lane-operations per second, of the
 * instructions the modular arithmetic is made of (register-only dependency chains, every SIMD full) and the rate of
 * a plain device-to-device copy of copy_bytes (bytes read + bytes written per second, best of three).  The benchmark
 * prints them beside the datasheet peaks; profiling runs use the copy as the kernel of known size that scales the
 * memory counters.  Synchronises the stream; allocates 2 GiB from the context's pool for the copy. */
typedef struct {
    double fma_f64, mul_f64, add_f64;  /* v_fma_f64, v_mul_f64, v_add_f64 */
    double rndne_add_f64;              /* v_rndne_f64 followed by v_add_f64, both counted */
    double mul_lo_u64, mul_hi_u64;     /* 64-bit integer multiply, low / high half (each with an add and a mask) */
    double copy_GBs;
    uint64_t copy_bytes;
    double clock_mhz;                  /* the device's nominal peak clock */
    uint32_t compute_units, reserved;
} hisa_calibration;
int hisa_calibrate(hisa_ctx* ctx, hisa_calibration* out);

/* The host-side check that every multiply-accumulate launch of the tensor kernels (Sec. "Runtime": convolution and
 * matrix multiplication over CipherTensors) passes before it reaches the GPU, callable on its own: no device, no
 * context, nothing is dereferenced.  A launch reads, per rotation amount ("tap"), batch * ic entries ct_words apart of
 * polys * limbs limbs of 2^log_n words, and writes batch * oc such entries; an optional second input (x2_extent != 0)
 * holds n_taps blocks x2_tap_words apart of batch * ic entries x2_words apart of lq limbs, its output batch * oc of
 * them; plaintext weights (w_extent != 0) are read at (T * w_stride_t + o * w_stride_oc) * w_words on limbs limbs
 * (w_words = 0: limbs * 2^log_n).  Every *_words / *_extent field counts the 8-byte words from the pointer the launch
 * would use to the end of its allocation; tap_words holds n_taps of them (null with n_taps = 1: tap0_words).
 * Inside the library the extents come from the context's allocator, so a launch whose shape fields do not match the
 * buffers behind its pointers is refused with HISA_ERR_ARG instead of running.
 * Returns HISA_OK when every access stays inside its allocation, HISA_ERR_ARG otherwise. */
typedef struct {
    int32_t n_taps, ic, oc, batch, log_n;
    int32_t limbs, polys, lq, gap;     /* polys: 2 (0 is read as 2) or 1; limbs >= lq use the primes gap further on */
    uint64_t ct_words;
    const uint64_t* tap_words;
    uint64_t tap0_words, out_words;
    uint64_t x2_tap_words, x2_words, x2_extent, out2_extent;
    uint64_t w_words, w_stride_t, w_stride_oc, w_extent;
} hisa_mac_extents;
int hisa_check_mac_extents(const hisa_mac_extents* a);

#ifdef __cplusplus
}
#endif
#endif /* HISA_H */
