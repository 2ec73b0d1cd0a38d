/*
 * cryptogen.h -- C ABI of the MI355X (gfx950) library for the server-side
 * ciphertext x ciphertext attention path of CryptoGen (BFV over
 * R_Q = Z_Q[X]/(X^N+1), Q a product of word-size primes).
 *
 * The library is keygen-free: no secret key, no encryption, no decryption.
 * It evaluates on ciphertexts that the caller already holds in device memory
 * (for instance PyTorch int64 tensors) and enqueues all work on the HIP stream
 * the caller passes.  It allocates device memory only in cg_create (constant
 * tables) and frees it in cg_destroy; every ciphertext, key, plaintext and
 * workspace buffer is allocated, owned and freed by the caller.
 *
 * Conventions shared by all entry points
 *   pointers    "dev" = device memory, "host" = host memory.  Device buffers
 *               must be 16-byte aligned.  stream is a hipStream_t passed as
 *               void* (NULL = the legacy default stream).
 *   ring element  uint64[k][N]: row i holds the canonical residues in [0,q_i)
 *               of the N coefficients (coefficient order, degree ascending).
 *   ciphertext  uint64[ncomp][k][N], ncomp = 2 (c0,c1) or 3 (d0,d1,d2).
 *   batch       `batch` ciphertexts are stored back to back; 1 <= batch <= 65536 units per
 *               call (an empty batch is CG_EINVAL, like any other invalid size).
 *   switch key  as generated: uint64[dnum][2][k+nsp][N], coefficient order,
 *               ciphertext primes first, then special primes (hybrid key
 *               switching, digit j = alpha consecutive ciphertext primes,
 *               key_j = (-a_j s + e_j + P T_j s', a_j) mod P Q).  It must be
 *               converted once with cg_ksk_prepare; the prepared form is
 *               opaque (cg_sizes.ksk_bytes bytes).
 *   results     every output residue is canonical, and is bit-identical to
 *               the definition over the integers stated at each entry point.
 *   errors      every call returns 0 or a negative cg_status; nothing throws,
 *               aborts or synchronises the device (except create/destroy).
 *               Invalid arguments are rejected before any kernel is launched.
 *   aliasing    outputs must not overlap inputs unless stated.
 *   threads     a context may be used from several host threads as long as
 *               concurrent calls use distinct workspaces; cg_decode_step,
 *               cg_decode_step_ext and cg_decode_step_hoisted use streams and events owned by the context,
 *               and cg_ntt_forward / cg_ntt_inverse an index table owned by it,
 *               so a context runs one of each of these at a time.
 *
 * Where the paper is cited: "section 4.3" is Auto-Regressive
 * Ciphertext-Ciphertext Multiplication (ARCC), "section 4.4" Encrypted
 * KV-Cache Management, "Algorithm 1" the appendix listing of noise refresh and
 * concatenation; the BFV scheme itself is only named there (section
 * "Cryptographic Libraries and Parameters"), so the arithmetic follows the
 * textbook Fan-Vercauteren definitions restated below.
 */
#ifndef CRYPTOGEN_H
#define CRYPTOGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cg_ctx cg_ctx;

typedef enum {
    CG_OK = 0,
    CG_EINVAL = -1,   /* null / misaligned pointer, bad size, unsupported parameter */
    CG_ENOMEM = -2,   /* table allocation failed in cg_create */
    CG_EHIP = -3,     /* a HIP runtime call or kernel launch reported an error */
    CG_ESCRATCH = -4  /* cg_mul_relin_static: the batch needs more scratch than the static array holds */
} cg_status;

typedef struct {
    uint32_t log2n;       /* ring degree N = 2^log2n, 12 <= log2n <= 14 */
    uint32_t k;           /* number of ciphertext primes, 1..6 */
    uint32_t nsp;         /* number of special (key-switching) primes, 1..2 */
    uint32_t alpha;       /* ciphertext primes per key-switch digit; divides k; <= min(3, nsp): with
                             fewer special primes than digit primes P < Q_j and every key switch
                             would add noise of the size of a whole prime */
    uint64_t t;           /* plaintext modulus, odd, < 2^20 */
    const uint64_t *q;    /* host: k distinct primes, q_i = 1 mod 2N, 2^40 < q_i < 2^50 */
    const uint64_t *p;    /* host: nsp primes, same conditions, distinct from q */
} cg_params;

typedef struct {
    size_t ct2_bytes;        /* one 2-component ciphertext */
    size_t ct3_bytes;        /* one 3-component ciphertext */
    size_t ksk_raw_bytes;    /* one switching key as generated */
    size_t ksk_bytes;        /* one prepared switching key */
    size_t plain_bytes;      /* one prepared plaintext (cg_plain_prepare output) */
    size_t ws_bytes_per_unit;/* workspace bytes per batch unit (see cg_workspace_bytes) */
    size_t ct_ext_bytes;     /* one ciphertext in transformed form (cg_cache_extend output) */
} cg_sizes;

/* Build a context: validates the parameters (CG_EINVAL otherwise), chooses the
 * library's private auxiliary primes, uploads twiddle and base-conversion
 * tables to the current device.  Synchronises the device. */
int cg_create(cg_ctx **out, const cg_params *prm);
int cg_destroy(cg_ctx *ctx);
int cg_get_sizes(const cg_ctx *ctx, cg_sizes *out);
/* Bytes of caller-provided scratch ("ws") that any call below needs for the
 * given batch; contents are undefined between calls. */
size_t cg_workspace_bytes(const cg_ctx *ctx, uint32_t batch);
const char *cg_strerror(int status);

/* Negacyclic number-theoretic transform of n_limbs ring rows, each modulo the
 * prime selected by prime_idx[i] (host array; 0..k-1 ciphertext primes,
 * k..k+nsp-1 special primes).  out[i][j] = in_i(psi^(2*bitrev(j)+1)) mod that
 * prime, psi its smallest primitive 2N-th root of unity; the inverse call
 * undoes it.  Canonical in, canonical out; in == out allowed.  Rows that follow the pattern
 * prime_idx[i] = i mod period need no table on the device; any other assignment is copied
 * from the host array when the call is made, which a graph replay would not repeat: on a
 * capturing stream that form returns CG_EINVAL.  This is the
 * transform every product below is built on (the paper's CT x CT cost is
 * dominated by it; it is not described there). */
int cg_ntt_forward(cg_ctx *ctx, void *stream, const uint64_t *in_dev, uint64_t *out_dev,
                   const uint32_t *prime_idx_host, uint32_t n_limbs);
int cg_ntt_inverse(cg_ctx *ctx, void *stream, const uint64_t *in_dev, uint64_t *out_dev,
                   const uint32_t *prime_idx_host, uint32_t n_limbs);

/* Switching key, as generated -> prepared form (once per key). */
int cg_ksk_prepare(cg_ctx *ctx, void *stream, const uint64_t *ksk_raw_dev, void *ksk_dev);

/* Plaintext polynomials (uint64[batch][N], coefficients in [0,t)) -> prepared
 * form used by cg_mul_plain / cg_kv_append: each coefficient is lifted to its
 * centred representative in (-t/2, t/2] before reduction mod every q_i. */
int cg_plain_prepare(cg_ctx *ctx, void *stream, const uint64_t *pt_dev, void *plain_dev,
                     uint32_t batch);

/* BFV tensor product with exact scaling (the "CT x CT multiplication" of
 * section 4.3, without relinearisation).  For unit u:
 *   a~, b~ = centred lifts of a[u / a_group], b[u] to Z[X]/(X^N+1);
 *   e0 = a~0 b~0, e1 = a~0 b~1 + a~1 b~0, e2 = a~1 b~1 over Z;
 *   out3[u] = (round(t e_i / Q) mod Q)_{i=0,1,2}   (nearest integer; no ties since Q is odd).
 * a holds ceil(batch / a_group) ciphertexts (a_group = 1: one per unit;
 * a_group = m: each a ciphertext is multiplied with m consecutive b's). */
int cg_mul(cg_ctx *ctx, void *stream, const uint64_t *a2_dev, const uint64_t *b2_dev,
           uint64_t *out3_dev, uint32_t batch, uint32_t a_group, void *ws_dev);

/* Sum of products with one scaling (the "accumulated" products of section 4.3 with the rounding
 * moved behind the sum): out3[g] = round(t/Q * sum_{i < group_len} a[g*group_len+i] (x) b[g*group_len+i])
 * mod Q, the tensor products (centred lifts, three components) summed over the integers before
 * the division.  a2_dev, b2_dev: n_groups * group_len ciphertexts each; out3_dev: n_groups
 * three-component results.  n_groups * group_len <= 65536.
 * ws_dev: cg_workspace_bytes(ctx, n_groups * group_len) bytes. */
int cg_mul_sum(cg_ctx *ctx, void *stream, const uint64_t *a2_dev, const uint64_t *b2_dev,
               uint64_t *out3_dev, uint32_t n_groups, uint32_t group_len, void *ws_dev);

/* Relinearisation: out2 = (d0 + u0, d1 + u1) with u = KeySwitch(d2, rlk):
 *   digit_j = d2 mod Q_j as the integer polynomial with coefficients in [0,Q_j);
 *   A_c = sum_j digit_j * key_{j,c}  mod P Q, coefficients taken in [0,PQ);
 *   u_c = floor((A_c + floor(P/2)) / P) mod Q.
 * out2 must not overlap in3. */
int cg_relin(cg_ctx *ctx, void *stream, const uint64_t *in3_dev, const void *rlk_dev,
             uint64_t *out2_dev, uint32_t batch, void *ws_dev);

/* cg_mul followed by cg_relin (same results as the two calls). */
int cg_mul_relin(cg_ctx *ctx, void *stream, const uint64_t *a2_dev, const uint64_t *b2_dev,
                 const void *rlk_dev, uint64_t *out2_dev, uint32_t batch, uint32_t a_group,
                 void *ws_dev);

/* cg_mul_relin for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and bit-identical results, but the scratch is an array of CG_STATIC_SCRATCH_BYTES
 * bytes that is part of the loaded library (every GPU the library is used on holds its own copy
 * until the process ends).  Neither this call nor anything below it allocates or frees memory.
 * A batch with cg_workspace_bytes(ctx, batch) > CG_STATIC_SCRATCH_BYTES is rejected with
 * CG_ESCRATCH before anything is launched (the limit is 9 products at N = 8192 with three
 * ciphertext primes, 28 at N = 4096 with two); the context's device must be the current one
 * (CG_EINVAL otherwise).  Every call on a GPU uses that GPU's one array: calls that overlap
 * in time on the same GPU -- from any context, stream or thread -- race on it and must be
 * ordered by the caller.  The array's previous contents never matter (every row is written
 * before it is read), so nothing is cleared. */
#define CG_STATIC_SCRATCH_BYTES (64u << 20)
size_t cg_static_scratch_bytes(void);
int cg_mul_relin_static(cg_ctx *ctx, void *stream, const uint64_t *a2_dev, const uint64_t *b2_dev,
                        const void *rlk_dev, uint64_t *out2_dev, uint32_t batch, uint32_t a_group);

/* Galois rotation (the "rotations" of the folding sum, section 4.3):
 * sigma_g moves the coefficient at index i to index i*g mod N, negated when
 * i*g mod 2N >= N;  rot = (sigma_g(c0) + u0, u1), u = KeySwitch(sigma_g(c1), gk).
 * galois_elt g must be odd, 0 < g < 2N, and gk the prepared key for s(X^g) -> s.
 * accumulate = 0: out2 = rot;  accumulate = 1: out2 = in2 + rot (one step of a
 * rotate-and-add reduction).  out2 must not overlap in2 (the permuted read of c0
 * happens while other outputs are written): any overlap of the two batch ranges is rejected. */
int cg_rotate(cg_ctx *ctx, void *stream, const uint64_t *in2_dev, uint32_t galois_elt,
              const void *gk_dev, uint64_t *out2_dev, uint32_t batch, int accumulate,
              void *ws_dev);

/* A series of rotations of the same ciphertexts (section 4.3 speaks of "a series of rotations";
 * this is the hoisted form, in which one decomposition of c1 serves the whole series):
 *   digit_j = c1 mod Q_j as the integer polynomial with coefficients in [0,Q_j), for every g the same;
 *   sigma_g acts on these integer polynomials (coefficient x at index i goes to index i*g mod N,
 *   as the negative integer -x when i*g mod 2N >= N);
 *   A_c = sum_j sigma_g(digit_j) * key^(g)_{j,c} mod P Q;  u_c = floor((A_c + floor(P/2)) / P) mod Q;
 *   out2[b][i] = (sigma_g(c0) + u0, u1) for g = galois_elts[i], key^(g) = gk[i].
 * The result decrypts to the same slots as cg_rotate's but is a different ciphertext (cg_rotate
 * lifts the digits of sigma_g(c1), where a negated coefficient is Q_j - x).  galois_elts_host /
 * gk_dev_host: host arrays of n_rot Galois elements (odd, < 2N) and device pointers to their
 * prepared keys; n_rot <= 4096 and batch * n_rot <= 65536.  out2: [batch][n_rot] ciphertexts, must
 * not overlap in2.  ws_dev: cg_workspace_bytes(ctx, batch * min(n_rot, 128) + batch) bytes. */
int cg_rotate_hoisted(cg_ctx *ctx, void *stream, const uint64_t *in2_dev, uint32_t n_rot,
                      const uint32_t *galois_elts_host, const void *const *gk_dev_host, uint64_t *out2_dev,
                      uint32_t batch, void *ws_dev);

/* A ciphertext plus a series of its rotations, with one division by P for the whole series (the
 * sums of rotated copies that section 4.3's products end in -- "rotations ... accumulated" --
 * regrouped so that several rotations act on the same ciphertext):
 *   digit_j and sigma_g on the digits as in cg_rotate_hoisted;
 *   A_c = sum_i sum_j sigma_{g_i}(digit_j) * key^(g_i)_{j,c} mod P Q;
 *   u_c = floor((A_c + floor(P/2)) / P) mod Q;
 *   out2[b] = (c0 + sum_i sigma_{g_i}(c0) + u0, c1 + u1).
 * It decrypts to the slot-wise sum of in2[b] and its n_rot rotations; it is not the sum of n_rot
 * separately rotated ciphertexts (those round n_rot times).  1 <= n_rot <= 128; arrays as in
 * cg_rotate_hoisted; out2 [batch] ciphertexts, must not overlap in2.
 * ws_dev: cg_workspace_bytes(ctx, batch) bytes. */
int cg_rotate_sum_hoisted(cg_ctx *ctx, void *stream, const uint64_t *in2_dev, uint32_t n_rot,
                          const uint32_t *galois_elts_host, const void *const *gk_dev_host,
                          uint64_t *out2_dev, uint32_t batch, void *ws_dev);

/* out = a + b component-wise mod q_i ("accumulated", section 4.3); ncomp = 2 or 3;
 * out may alias a or b. */
int cg_add(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *b_dev,
           uint64_t *out_dev, uint32_t ncomp, uint32_t batch);

/* Ciphertext +- plaintext (the server's two moves of the lazy noise refresh, Algorithm 1 step 1:
 * the share cache - r goes to the client, r is added back to what returns):
 *   out2[u] = (c0 +- floor(Q/t) * pt[u mod n_plain], c1),  pt coefficients in [0,t),
 * floor(Q/t) being the scale at which an encryption carries its plaintext.  negative != 0
 * subtracts.  pt_dev: uint64[n_plain][N] plaintext polynomials (not prepared); out2 may alias in2. */
int cg_add_plain(cg_ctx *ctx, void *stream, const uint64_t *in2_dev, const uint64_t *pt_dev,
                 uint32_t n_plain, int negative, uint64_t *out2_dev, uint32_t batch);

/* Ciphertext x plaintext (MultPlain of Algorithm 1): out2[u] = in2[u] * plain[u * plain_stride]
 * in R_Q, the plaintext lifted centred (see cg_plain_prepare).  plain_stride = 0
 * applies one plaintext to the whole batch. */
int cg_mul_plain(cg_ctx *ctx, void *stream, const uint64_t *in2_dev, const void *plain_dev,
                 uint32_t plain_stride, uint64_t *out2_dev, uint32_t batch, void *ws_dev);

/* Slot-aware concatenation into the packed cache (Algorithm 1, steps 2-3; section 4.4).
 * For each of n_caches independent caches c (e.g. heads x {K,V}):
 *   B = N / d2 tokens per cache ciphertext; token index tau (0-based, same for all caches);
 *   cache c occupies cache_dev + c * cache_stride_cts ciphertexts;
 *   cache[c][tau / B] <- cache[c][tau / B] + rows[c] * masks[tau mod B]      (in R_Q)
 * where masks_dev holds the B prepared block-mask plaintexts (block b selects flat
 * slots [b d2, (b+1) d2)) and rows[c] is the new d2-vector tiled into all B blocks.
 * When tau mod B == 0 the target ciphertext is treated as all-zero (it is opened
 * by this call; its previous contents are ignored).  Returns CG_EINVAL if
 * tau / B >= cache_stride_cts. */
int cg_kv_append(cg_ctx *ctx, void *stream, uint64_t *cache_dev, uint32_t cache_stride_cts,
                 uint32_t n_caches, uint32_t tau, const uint64_t *rows_dev,
                 const void *masks_dev, uint32_t d2, void *ws_dev);

/* Decode attention scores, ARCC inner-outer mode (section 4.3): for every head h
 * and cache ciphertext c < n_cts (head h's cache starts at ciphertext index
 * h * cache_stride_cts of kcache_dev, the layout cg_kv_append maintains):
 *   x = relin(mul(q[h], K[h][c]));  for sh = 1, 2, 4, ..., d2/2: x = x + rotate(x, 3^sh mod 2N);
 *   out[h][c] = x  -- flat slot b*d2 of x decrypts to <q_h, K_token b> mod t.
 * out is dense: [heads][n_cts] ciphertexts.
 * gk_fold_dev_host: host array of log2(d2) device pointers, prepared keys for
 * g = 3^1, 3^2, 3^4, ... (mod 2N) in that order. */
int cg_decode_scores(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *kcache_dev,
                     uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                     const void *rlk_dev,
                     const void *const *gk_fold_dev_host, uint64_t *out_dev, void *ws_dev);

/* Decode attention context, ARCC inner-inner mode with the weight of token b
 * already broadcast over block b (section 4.3): for every head h
 *   y = sum_c mul(a[h][c], V[h][c])   (three components, c ascending);  x = relin(y);
 *   for sh = d2, 2 d2, ..., N/4: x = x + rotate(x, 3^sh mod 2N);  x = x + rotate(x, 2N-1);
 *   out[h] = x  -- every block of x decrypts to sum_tokens a_tau V_tau mod t.
 * a is dense ([heads][n_cts]); head h's V cache starts at ciphertext index
 * h * cache_stride_cts of vcache_dev.
 * gk_block_dev_host: host array of device pointers, prepared keys for
 * g = 3^d2, 3^(2 d2), ..., 3^(N/4), then 2N-1, in that order. */
int cg_decode_context(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *vcache_dev,
                      uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                      const void *rlk_dev,
                      const void *const *gk_block_dev_host, uint64_t *out_dev, void *ws_dev);

/* One decode step of one layer over the encrypted cache (Algorithm 1 steps 2-3 followed by the
 * two products of section 4.3): equivalent to
 *   cg_kv_append(cache, cache_stride_cts, 2*heads, tau, rows, masks, d2);
 *   cg_decode_scores (q, K caches, heads, n_cts, ...) -> scores_dev  [heads][n_cts];
 *   cg_decode_context(a, V caches, heads, n_cts, ...) -> context_dev [heads];
 * with cache_dev holding the heads K caches followed by the heads V caches (each
 * cache_stride_cts ciphertexts) and rows_dev the new K rows followed by the new V rows.
 * The appended ciphertext is visible to the products when tau / (N/d2) < n_cts.
 * Independent branches run side by side on two internal streams (default priority) that
 * fork from and join back into `stream`, so the call is ordered on `stream` like any other;
 * results are bit-identical to the three calls in sequence.  A context runs one such call
 * at a time.  ws_dev: cg_decode_step_workspace_bytes(ctx, heads, n_cts) bytes. */
size_t cg_decode_step_workspace_bytes(const cg_ctx *ctx, uint32_t heads, uint32_t n_cts);
int cg_decode_step(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *a_dev,
                   uint64_t *cache_dev, uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts,
                   uint32_t d2, uint32_t tau, const uint64_t *rows_dev, const void *masks_dev,
                   const void *rlk_dev, const void *const *gk_fold_dev_host,
                   const void *const *gk_block_dev_host, uint64_t *scores_dev, uint64_t *context_dev,
                   void *ws_dev);

/* The decode products with their folding sums taken in rounds (section 4.3 fixes what is summed --
 * the d2 slots of a block for the scores, the N/d2 blocks for the context -- not the order).  The
 * rotate-and-add chain applies generators g_0 .. g_{B-1} one after the other (scores: g_b =
 * 3^(2^b), B = log2 d2; context: g_b = 3^(d2 2^b) for b < log2(N/(2 d2)), then 2N-1), each step on
 * the previous step's result.  Here the B bits are cut into R = ceil(B / round_bits) chunks, as
 * even as possible, the longer ones first; round r over bits [b0, b0 + c) is one
 * cg_rotate_sum_hoisted of the previous round's result with the 2^c - 1 Galois elements
 *   e_m = product of g_(b0+i) over the bits i set in m,  m = 1 .. 2^c - 1  (in this order),
 * so R dependent key switches replace B.  Everything before the folding sum (products, the sum
 * over cache ciphertexts, the relinearisation) is as in cg_decode_scores / cg_decode_context, and
 * the results decrypt to the same slots; they are other ciphertexts.  1 <= round_bits <= 7.
 * gk_rounds_dev_host: host array of device pointers to the prepared keys of all rounds, round 0's
 * 2^c - 1 keys first.  kext_dev / vext_dev: the cache's transformed form (cg_cache_extend) or
 * NULL; when given, kc_dev / vc_dev is not read and may be NULL.  sum_before_scaling (0 or 1,
 * context only): 1 = the n_cts products of a head are summed as tensor products over the integers
 * and scaled by t/Q once (cg_mul_sum) instead of scaled one by one and added -- one rounding
 * instead of n_cts, again other bits for the same slots.  cg_decode_step_hoisted is
 * cg_decode_step (cache_ext_dev NULL) or cg_decode_step_ext with both folding sums in rounds.
 * Workspaces as for the calls they replace. */
/* The Galois elements of all rounds in the order of gk_rounds_dev_host, for the scores' folding
 * sum (which = 0) or the context's (which = 1): writes min(cap, n) of them to elts_host and n to
 * n_out (host memory; no device work). */
int cg_round_galois(const cg_ctx *ctx, int which, uint32_t d2, uint32_t round_bits, uint32_t *elts_host,
                    uint32_t cap, uint32_t *n_out);
int cg_decode_scores_hoisted(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *kc_dev,
                             const void *kext_dev, uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts,
                             uint32_t d2, uint32_t round_bits, const void *rlk_dev,
                             const void *const *gk_rounds_dev_host, uint64_t *out_dev, void *ws_dev);
int cg_decode_context_hoisted(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *vc_dev,
                              const void *vext_dev, uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts,
                              uint32_t d2, uint32_t round_bits, int sum_before_scaling, const void *rlk_dev,
                              const void *const *gk_rounds_dev_host, uint64_t *out_dev, void *ws_dev);
int cg_decode_step_hoisted(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *a_dev,
                           uint64_t *cache_dev, void *cache_ext_dev, uint32_t heads, uint32_t n_cts,
                           uint32_t cache_stride_cts, uint32_t d2, uint32_t tau, const uint64_t *rows_dev,
                           const void *masks_dev, const void *rlk_dev, uint32_t fold_round_bits,
                           const void *const *gk_fold_rounds_dev_host, uint32_t block_round_bits,
                           int sum_before_scaling, const void *const *gk_block_rounds_dev_host,
                           uint64_t *scores_dev, uint64_t *context_dev, void *ws_dev);

/* The cache kept in transformed form (an optimisation of the decode scan that leaves every
 * result bit-identical): a ciphertext that is multiplied in many steps -- every cache
 * ciphertext is -- need not be lifted to the extended basis and transformed again each time.
 * cg_cache_extend writes, for ciphertext (g, i), g < n_groups, i < group_len, at index
 * g * group_stride_cts + i of cts_dev, its transformed form (opaque, cg_sizes.ct_ext_bytes
 * bytes) at the same index of ext_dev.  cg_decode_scores_ext / cg_decode_context_ext are
 * cg_decode_scores / cg_decode_context reading that form (same cache geometry, indices in
 * units of transformed ciphertexts).  cg_decode_step_ext is cg_decode_step with the
 * transformed copy of the whole cache ([2*heads][cache_stride_cts], K caches first) beside
 * it: the products read the copy, and after the append the copy of the ciphertext each
 * cache received is refreshed (the untransformed cache stays authoritative and is what the
 * append updates).  The copy must be up to date for every ciphertext the products read. */
int cg_cache_extend(cg_ctx *ctx, void *stream, const uint64_t *cts_dev, uint32_t n_groups,
                    uint32_t group_len, uint32_t group_stride_cts, void *ext_dev);
int cg_decode_scores_ext(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const void *kext_dev,
                         uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                         const void *rlk_dev, const void *const *gk_fold_dev_host, uint64_t *out_dev,
                         void *ws_dev);
int cg_decode_context_ext(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const void *vext_dev,
                          uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                          const void *rlk_dev, const void *const *gk_block_dev_host, uint64_t *out_dev,
                          void *ws_dev);
int cg_decode_step_ext(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *a_dev,
                       uint64_t *cache_dev, void *cache_ext_dev, uint32_t heads, uint32_t n_cts,
                       uint32_t cache_stride_cts, uint32_t d2, uint32_t tau, const uint64_t *rows_dev,
                       const void *masks_dev, const void *rlk_dev, const void *const *gk_fold_dev_host,
                       const void *const *gk_block_dev_host, uint64_t *scores_dev, uint64_t *context_dev,
                       void *ws_dev);

/* Decode attention scores against an outer-packed cache segment (one ciphertext per feature
 * column: kcols[h][j] holds K[tau][j] in flat slot tau), ARCC inner-inner mode (section 4.3 and
 * its figure on masking and rotating a scalar).  q[h] is the query tiled with period d2.  For
 * every head h and feature j < d2:
 *   x_j = q[h] * mask_j           (ct x pt; mask_j = prepared plaintext selecting slots = j mod d2)
 *   for sh = 1, 2, 4, ..., d2/2:  x_j = x_j + rotate(x_j, 3^sh mod 2N)      -> every slot holds q_j
 *   y = y + mul(x_j, kcols[h][j])                                 (three components, j ascending)
 * out[h] = relin(y)  -- flat slot tau decrypts to <q_h, K_tau> mod t.
 * masks_dev: d2 prepared plaintexts (cg_plain_prepare) in order j = 0..d2-1; gk_fold as in
 * cg_decode_scores; the workspace must be sized for heads * d2 units. */
int cg_decode_scores_outer(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *kcols_dev,
                           uint32_t heads, uint32_t d2, const void *masks_dev, const void *rlk_dev,
                           const void *const *gk_fold_dev_host, uint64_t *out_dev, void *ws_dev);

/* Decode attention context against an outer-packed value segment (vcols[h][j] holds V[tau][j] in
 * flat slot tau), ARCC inner-outer mode (section 4.3): a[h] holds the weight a_tau in flat slot tau.
 * For every head h and feature j < d2:
 *   x = relin(mul(a[h], vcols[h][j]));
 *   for sh = 1, 2, 4, ..., N/4: x = x + rotate(x, 3^sh mod 2N);  x = x + rotate(x, 2N-1);
 *   out[h][j] = x  -- every slot decrypts to o_j = sum_tau a_tau V[tau][j] mod t.
 * gk_all_dev_host: prepared keys for g = 3^1, 3^2, 3^4, ..., 3^(N/4), then 2N-1 (log2(N/2) + 1 keys).
 * d2 may be any positive column count; the workspace must be sized for heads * d2 units. */
int cg_decode_context_outer(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *vcols_dev,
                            uint32_t heads, uint32_t d2, const void *rlk_dev,
                            const void *const *gk_all_dev_host, uint64_t *out_dev, void *ws_dev);

/* Prefill Q K^T for `heads` heads as m = N/d2 generalised diagonals per head
 * (the paper's outer-outer CT x CT product is named, not specified; this is the
 * library's documented procedure).  Q and K are token-major row-packed
 * (token i in block i).  With H = m/2:  K_0 = K, K_r = rotate(K_{r-1}, 3^d2);
 * for sigma in {0,1}, r in [0,H): K' = K_r (sigma = 0) or rotate(K_r, 2N-1);
 * x = relin(mul(Q, K')); folding sum as in cg_decode_scores;
 * out[h][sigma*H + r] = x.  gk_fold as in cg_decode_scores; gk_blk = key for
 * 3^d2, gk_swap = key for 2N-1. */
int cg_prefill_qk(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *k_dev,
                  uint32_t heads, uint32_t d2, const void *rlk_dev,
                  const void *const *gk_fold_dev_host, const void *gk_blk_dev,
                  const void *gk_swap_dev, uint64_t *out_dev, void *ws_dev);

/* Prefill context O = A V for every head (the softmax-times-values product of the prompt,
 * section 4.1 "outer-outer"; the paper gives no procedure -- this is the product over the same
 * generalised diagonals as cg_prefill_qk).  v_dev: [heads] token-major ciphertexts (token i in
 * block i, the layout cg_kv_append builds); a_dev: [heads][m] ciphertexts, m = N/d2, unit
 * (sigma, r) = sigma*H + r (H = m/2) holding A[i][j(i,sigma,r)] in all d2 slots of block i, with
 * j as in cg_prefill_qk.  Computes, per head, the rotated copies V_(sigma,r) exactly as
 * cg_prefill_qk does for K, y = sum over units of mul(a[h][u], V_u) (three components, u
 * ascending), out[h] = relin(y): block i of out[h] decrypts to sum_j A[i][j] V[j][:] mod t.
 * gk_blk / gk_swap: prepared keys for 3^d2 and 2N-1. */
int cg_prefill_av(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *v_dev,
                  uint32_t heads, uint32_t d2, const void *rlk_dev, const void *gk_blk_dev,
                  const void *gk_swap_dev, uint64_t *out_dev, void *ws_dev);

/* cg_prefill_qk / cg_prefill_av with the m - 1 rotated copies of K (of V) made as one series of
 * hoisted rotations of K (V) itself (cg_rotate_hoisted) instead of m/2 - 1 successive block
 * rotations and m/2 row swaps: copy sigma*H + r is rotate_hoisted(K, g), g = 3^(d2 r) mod 2N for
 * sigma = 0 and (2N-1) 3^(d2 r) mod 2N for sigma = 1; everything after the copies is unchanged.
 * The outputs decrypt to the same values as the unhoisted calls' but are other ciphertexts (each
 * copy has seen one key switch instead of up to m/2).  gk_copies_dev_host: host array of m - 1
 * device pointers, prepared keys of copies 1 .. m-1 in that order.  fold_round_bits = 0: the
 * folding sum as in cg_prefill_qk (gk_fold as there); >= 1: in rounds of that many bits as in
 * cg_decode_scores_hoisted, gk_fold_dev_host then holding the rounds' keys in its order.
 * sum_before_scaling (cg_prefill_av_hoisted, 0 or 1): 1 = the m products of a head summed as
 * tensor products and scaled once (cg_mul_sum) instead of scaled one by one and added. */
int cg_prefill_qk_hoisted(cg_ctx *ctx, void *stream, const uint64_t *q_dev, const uint64_t *k_dev,
                          uint32_t heads, uint32_t d2, uint32_t fold_round_bits, const void *rlk_dev,
                          const void *const *gk_fold_dev_host, const void *const *gk_copies_dev_host,
                          uint64_t *out_dev, void *ws_dev);
int cg_prefill_av_hoisted(cg_ctx *ctx, void *stream, const uint64_t *a_dev, const uint64_t *v_dev,
                          uint32_t heads, uint32_t d2, int sum_before_scaling, const void *rlk_dev,
                          const void *const *gk_copies_dev_host, uint64_t *out_dev, void *ws_dev);

/* Compaction of the m score ciphertexts of cg_prefill_qk, whose useful values sit in slot 0 of
 * every block (a step the score hand-over to the non-linear protocol needs; not described in
 * the paper).  Units come in groups of w = min(d2, H) consecutive diagonals; every unit is
 * multiplied by mask0 (prepared plaintext selecting slot 0 of each block) and the group is
 * summed with diagonal r' of the group shifted right by r' slots, as a pairwise tree: at
 * level l = 0, 1, ..., log2(w)-1:  y[j 2^(l+1)] += rotate(y[j 2^(l+1) + 2^l], 3^(N/2 - 2^l)).
 * out_dev: [heads * m / w] ciphertexts; slot i*d2 + r' of group output g holds the useful
 * value of diagonal g*w + r' for token i.  x_dev is not modified.
 * gk_right_dev_host: host array of log2(w) device pointers, prepared keys for
 * g = 3^(N/2 - 1), 3^(N/2 - 2), 3^(N/2 - 4), ... (mod 2N) in that order. */
int cg_prefill_repack(cg_ctx *ctx, void *stream, const uint64_t *x_dev, uint32_t heads, uint32_t d2,
                      const void *mask0_dev, const void *const *gk_right_dev_host, uint64_t *out_dev,
                      void *ws_dev);

/* Ciphertext x plaintext vector-matrix product of the decode step (section 4.2, "inner-diagonal
 * CPVM": one token in one ciphertext, about d1 d2 / N plaintext products and O(log) rotations per
 * matrix, cost independent of the prompt length; the paper states the operation and these counts,
 * the procedure is this library's):
 *   y[u] = x W_u  for u < units, every W_u a d1 x d2 plaintext matrix given as n_diag diagonals.
 * Layout (D1 = tile length: the power of two >= max(d1, d2, N/d2), at most N/2; T = N/D1 tiles;
 * n_diag = d2 / T): x_dev is one ciphertext whose flat slot r D1 + i holds feature
 * (i + n_diag r) mod D1 of the token (zero beyond d1); diagonal c of a matrix holds at flat slot
 * s the entry W[f][s mod d2], f being the feature that slot s of x shows after a left rotation by c
 * (zero for f >= d1).  diags_dev: prepared plaintexts (cg_plain_prepare) [units][n_diag].
 * Procedure: copies x_c = rotate(x, 3^c), c < n_diag, by a doubling tree (copy 2^l + i = copy i
 * rotated by 3^(2^l)); y[u] = sum_c x_c * diag[u][c]; then y += rotate(y, g) for g = 3^d2, 3^(2 d2),
 * ..., 3^(N/4), 2N-1.  Every slot s of out_dev[u] then decrypts to (x W_u)[s mod d2] mod t: the
 * layout cg_decode_scores takes its query in and cg_kv_append its new row.
 * gk_shift_dev_host: host array of log2(n_diag) device pointers, prepared keys for 3^1, 3^2,
 * 3^4, ... (may be NULL when n_diag is 1); gk_block_dev_host: as for cg_decode_context.
 * n_diag: a power of two, at most min(d2, 64).  out_dev: [units] ciphertexts, must not overlap
 * x_dev.  ws_dev: cg_workspace_bytes(ctx, units + n_diag) bytes. */
int cg_cpvm(cg_ctx *ctx, void *stream, const uint64_t *x_dev, const void *diags_dev, uint32_t units,
            uint32_t n_diag, uint32_t d2, const void *const *gk_shift_dev_host,
            const void *const *gk_block_dev_host, uint64_t *out_dev, void *ws_dev);

/* cg_cpvm with the n_diag - 1 rotated copies of the token made as one series of hoisted rotations
 * of the token (copy c = rotate_hoisted(x, 3^c)) instead of the doubling tree: n_diag - 1 keys
 * instead of log2(n_diag), one decomposition instead of n_diag - 1.  gk_copies_dev_host: prepared
 * keys for 3^1, 3^2, ..., 3^(n_diag - 1) (may be NULL when n_diag is 1).  block_round_bits = 0:
 * the sum over residue classes as in cg_cpvm (gk_block as there); >= 1: in rounds of that many
 * bits as in cg_decode_context_hoisted, gk_block_dev_host then holding the rounds' keys in its
 * order (cg_round_galois, which = 1). */
int cg_cpvm_hoisted(cg_ctx *ctx, void *stream, const uint64_t *x_dev, const void *diags_dev, uint32_t units,
                    uint32_t n_diag, uint32_t d2, uint32_t block_round_bits,
                    const void *const *gk_copies_dev_host, const void *const *gk_block_dev_host,
                    uint64_t *out_dev, void *ws_dev);

#ifdef __cplusplus
}
#endif
#endif /* CRYPTOGEN_H */
