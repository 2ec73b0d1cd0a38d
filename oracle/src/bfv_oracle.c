/*
 * CPU oracle for the encrypted-attention hot path (BFV over Z[X]/(X^N+1)).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is compared against; it shares no code, header, table or
 * constant with the HIP path and nothing in the product path may call it.
 *
 * Every evaluator operation is written as its definition over the integers
 * (Fan-Vercauteren BFV; the paper names the scheme in its section
 * "Cryptographic Libraries and Parameters" and treats it as a black box):
 *
 *   mul       lift both ciphertexts to centred integer polynomials, form the
 *             three tensor components over Z, scale each coefficient by t/Q
 *             and round to nearest, reduce mod Q.
 *   keyswitch hybrid key switching: split the input in digits modulo groups of
 *             alpha ciphertext primes (non-centred representatives), multiply
 *             by the switching key modulo P*Q, divide by P with rounding.
 *   relin     (d0,d1,d2) -> (d0,d1) + keyswitch(d2, rlk)
 *   rotate    Galois map X -> X^g on both components, then key switch the
 *             second one (the paper's "rotations", section 4.3).
 *   add, mul_plain (centred plaintext lift) -- used by the cache append,
 *             Algorithm 1 of the paper's appendix.
 *
 * Polynomial products are the one place a fast primitive is used as a step: a
 * textbook radix-2 number-theoretic transform per word-size prime (checked
 * against the schoolbook convolution in the tests).  Integer (not modular)
 * products are obtained by multiplying modulo enough private 61-bit primes and
 * reconstructing with the Chinese remainder theorem into a small fixed-size
 * big integer, on which the rounding divisions are done exactly (schoolbook
 * long division).  Word-size modular products use the compiler's 128-bit
 * integer remainder; nothing here is tuned.
 *
 * Layouts: a ring element modulo Q is uint64[k][N] (one row of canonical
 * residues per ciphertext prime, coefficient order); a ciphertext is
 * uint64[ncomp][k][N]; a switching key is uint64[dnum][2][k+nsp][N] with the
 * ciphertext primes first, then the special primes.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint64_t u64;
typedef uint32_t u32;
typedef unsigned __int128 u128;

/* ------------------------------------------------------------------ */
/* word-size modular arithmetic                                        */
/* ------------------------------------------------------------------ */
static u64 mulmod(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
static u64 addmod(u64 a, u64 b, u64 m) { u64 s = a + b; return s >= m ? s - m : s; }
static u64 submod(u64 a, u64 b, u64 m) { return a >= b ? a - b : a + m - b; }
static u64 powmod(u64 a, u64 e, u64 m)
{
    u64 r = 1 % m;
    a %= m;
    while (e) {
        if (e & 1) r = mulmod(r, a, m);
        a = mulmod(a, a, m);
        e >>= 1;
    }
    return r;
}
static u64 invmod_prime(u64 a, u64 m) { return powmod(a, m - 2, m); }

/* deterministic Miller-Rabin for 64-bit integers */
static int is_prime_u64(u64 n)
{
    static const u64 bases[12] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
    if (n < 2) return 0;
    for (int i = 0; i < 12; i++) {
        if (n == bases[i]) return 1;
        if (n % bases[i] == 0) return 0;
    }
    u64 d = n - 1;
    int s = 0;
    while ((d & 1) == 0) { d >>= 1; s++; }
    for (int i = 0; i < 12; i++) {
        u64 x = powmod(bases[i], d, n);
        if (x == 1 || x == n - 1) continue;
        int comp = 1;
        for (int r = 1; r < s; r++) {
            x = mulmod(x, x, n);
            if (x == n - 1) { comp = 0; break; }
        }
        if (comp) return 0;
    }
    return 1;
}

/* smallest primitive 2N-th root of unity modulo the prime m (m = 1 mod 2N) */
u64 orc_min_psi(int N, u64 m)
{
    u64 two_n = 2 * (u64)N;
    u64 root = 0;
    for (u64 x = 2; x < m; x++) {
        u64 r = powmod(x, (m - 1) / two_n, m);
        if (powmod(r, (u64)N, m) == m - 1) { root = r; break; }
    }
    /* all primitive roots are the odd powers of any one of them */
    u64 best = root, cur = root, sq = mulmod(root, root, m);
    for (int i = 1; i < N; i++) {
        cur = mulmod(cur, sq, m);
        if (cur < best) best = cur;
    }
    return best;
}

/* ------------------------------------------------------------------ */
/* textbook transforms                                                  */
/* ------------------------------------------------------------------ */
static unsigned bitrev(unsigned x, int bits)
{
    unsigned r = 0;
    for (int i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}
static int ilog2(int n) { int l = 0; while ((1 << l) < n) l++; return l; }

/* in-place cyclic DFT of length n (power of two): x[i] <- sum_j x[j] w^(ij),
 * natural order in and out; w has order n modulo m. */
static void dft_pow2(u64 *x, int n, u64 w, u64 m)
{
    int lg = ilog2(n);
    for (int i = 0; i < n; i++) {
        int j = (int)bitrev((unsigned)i, lg);
        if (i < j) { u64 tmp = x[i]; x[i] = x[j]; x[j] = tmp; }
    }
    for (int len = 2; len <= n; len <<= 1) {
        u64 wl = powmod(w, (u64)(n / len), m);
        for (int i = 0; i < n; i += len) {
            u64 wk = 1;
            for (int j = 0; j < len / 2; j++) {
                u64 u = x[i + j];
                u64 v = mulmod(x[i + j + len / 2], wk, m);
                x[i + j] = addmod(u, v, m);
                x[i + j + len / 2] = submod(u, v, m);
                wk = mulmod(wk, wl, m);
            }
        }
    }
}

/* out[i] = a(psi^(2i+1)), i = 0..N-1 (natural order) */
void orc_eval_odd(const u64 *a, u64 *out, int N, u64 m, u64 psi)
{
    u64 pw = 1;
    for (int i = 0; i < N; i++) {
        out[i] = mulmod(a[i] % m, pw, m);
        pw = mulmod(pw, psi, m);
    }
    dft_pow2(out, N, mulmod(psi, psi, m), m);
}

/* inverse of orc_eval_odd */
void orc_interp_odd(const u64 *ev, u64 *a, int N, u64 m, u64 psi)
{
    u64 ipsi = invmod_prime(psi, m);
    u64 iw = mulmod(ipsi, ipsi, m);
    u64 in = invmod_prime((u64)N % m, m);
    for (int i = 0; i < N; i++) a[i] = ev[i] % m;
    dft_pow2(a, N, iw, m);
    u64 pw = in;
    for (int i = 0; i < N; i++) {
        a[i] = mulmod(a[i], pw, m);
        pw = mulmod(pw, ipsi, m);
    }
}

/* negacyclic product c = a*b in Z_m[X]/(X^N+1); psi = any primitive 2N-th root */
static void polymul_psi(const u64 *a, const u64 *b, u64 *c, int N, u64 m, u64 psi)
{
    u64 *ea = (u64 *)malloc(sizeof(u64) * (size_t)N * 2);
    u64 *eb = ea + N;
    orc_eval_odd(a, ea, N, m, psi);
    orc_eval_odd(b, eb, N, m, psi);
    for (int i = 0; i < N; i++) ea[i] = mulmod(ea[i], eb[i], m);
    orc_interp_odd(ea, c, N, m, psi);
    free(ea);
}

void orc_polymul(const u64 *a, const u64 *b, u64 *c, int N, u64 m)
{
    polymul_psi(a, b, c, N, m, orc_min_psi(N, m));
}

/* The transform the device library exposes: psi = smallest primitive 2N-th
 * root, output index i holds a(psi^(2*bitrev(i)+1)). */
void orc_ntt_forward(const u64 *a, u64 *out, int N, u64 m)
{
    u64 *ev = (u64 *)malloc(sizeof(u64) * (size_t)N);
    orc_eval_odd(a, ev, N, m, orc_min_psi(N, m));
    int lg = ilog2(N);
    for (int i = 0; i < N; i++) out[i] = ev[bitrev((unsigned)i, lg)];
    free(ev);
}
void orc_ntt_inverse(const u64 *in, u64 *a, int N, u64 m)
{
    u64 *ev = (u64 *)malloc(sizeof(u64) * (size_t)N);
    int lg = ilog2(N);
    for (int i = 0; i < N; i++) ev[bitrev((unsigned)i, lg)] = in[i];
    orc_interp_odd(ev, a, N, m, orc_min_psi(N, m));
    free(ev);
}

/* ------------------------------------------------------------------ */
/* small fixed-capacity unsigned big integers, base 2^32                */
/* ------------------------------------------------------------------ */
#define BN_CAP 72
typedef struct { int n; u32 w[BN_CAP]; } bn;

static void bn_norm(bn *a) { while (a->n > 0 && a->w[a->n - 1] == 0) a->n--; }
static void bn_set_u64(bn *a, u64 v)
{
    a->n = 0;
    if (v) {
        a->w[0] = (u32)v;
        a->w[1] = (u32)(v >> 32);
        a->n = a->w[1] ? 2 : 1;
    }
}
static int bn_cmp(const bn *a, const bn *b)
{
    if (a->n != b->n) return a->n < b->n ? -1 : 1;
    for (int i = a->n - 1; i >= 0; i--)
        if (a->w[i] != b->w[i]) return a->w[i] < b->w[i] ? -1 : 1;
    return 0;
}
static void bn_add(bn *r, const bn *a, const bn *b)
{
    int n = a->n > b->n ? a->n : b->n;
    u64 c = 0;
    for (int i = 0; i < n; i++) {
        u64 s = c + (i < a->n ? a->w[i] : 0) + (i < b->n ? b->w[i] : 0);
        r->w[i] = (u32)s;
        c = s >> 32;
    }
    r->n = n;
    if (c) r->w[r->n++] = (u32)c;
}
/* r = a - b, requires a >= b */
static void bn_sub(bn *r, const bn *a, const bn *b)
{
    int64_t br = 0;
    for (int i = 0; i < a->n; i++) {
        int64_t d = (int64_t)a->w[i] - (i < b->n ? (int64_t)b->w[i] : 0) - br;
        br = d < 0;
        r->w[i] = (u32)d;
    }
    r->n = a->n;
    bn_norm(r);
}
/* r = a*b, r distinct from a and b */
static void bn_mul(bn *r, const bn *a, const bn *b)
{
    if (a->n == 0 || b->n == 0) { r->n = 0; return; }
    int n = a->n + b->n;
    for (int i = 0; i < n; i++) r->w[i] = 0;
    for (int i = 0; i < a->n; i++) {
        u64 c = 0;
        for (int j = 0; j < b->n; j++) {
            u64 s = (u64)a->w[i] * b->w[j] + r->w[i + j] + c;
            r->w[i + j] = (u32)s;
            c = s >> 32;
        }
        r->w[i + b->n] = (u32)c;
    }
    r->n = n;
    bn_norm(r);
}
static void bn_mul_u64(bn *r, const bn *a, u64 m)
{
    bn mm;
    bn_set_u64(&mm, m);
    bn_mul(r, a, &mm);
}
static u64 bn_mod_u64(const bn *a, u64 m)
{
    u64 r = 0;
    for (int i = a->n - 1; i >= 0; i--)
        r = (u64)((((u128)r << 32) | a->w[i]) % m);
    return r;
}
static void bn_shr1(bn *a)
{
    for (int i = 0; i < a->n; i++) {
        u32 hi = (i + 1 < a->n) ? a->w[i + 1] : 0;
        a->w[i] = (a->w[i] >> 1) | (hi << 31);
    }
    bn_norm(a);
}
static void bn_shl1(bn *a)
{
    u32 c = 0;
    for (int i = 0; i < a->n; i++) {
        u32 nc = a->w[i] >> 31;
        a->w[i] = (a->w[i] << 1) | c;
        c = nc;
    }
    if (c) a->w[a->n++] = c;
}
/* schoolbook long division (Knuth, algorithm D): a = q*b + r, 0 <= r < b, b != 0 */
static void bn_divmod(bn *q, bn *r, const bn *a, const bn *b)
{
    if (bn_cmp(a, b) < 0) { bn t = *a; q->n = 0; *r = t; return; }
    if (b->n == 1) {
        u64 rem = 0;
        bn qq;
        qq.n = a->n;
        for (int i = a->n - 1; i >= 0; i--) {
            u64 cur = (rem << 32) | a->w[i];
            qq.w[i] = (u32)(cur / b->w[0]);
            rem = cur % b->w[0];
        }
        bn_norm(&qq);
        *q = qq;
        bn_set_u64(r, rem);
        return;
    }
    const u64 base = (u64)1 << 32;
    int n = b->n, m = a->n;
    int s = __builtin_clz(b->w[n - 1]);
    u32 vn[BN_CAP], un[BN_CAP + 1];
    for (int i = n - 1; i > 0; i--)
        vn[i] = (b->w[i] << s) | (s ? (b->w[i - 1] >> (32 - s)) : 0);
    vn[0] = b->w[0] << s;
    un[m] = s ? (a->w[m - 1] >> (32 - s)) : 0;
    for (int i = m - 1; i > 0; i--)
        un[i] = (a->w[i] << s) | (s ? (a->w[i - 1] >> (32 - s)) : 0);
    un[0] = a->w[0] << s;
    bn qq;
    for (int j = m - n; j >= 0; j--) {
        u64 num = ((u64)un[j + n] << 32) | un[j + n - 1];
        u64 qhat = num / vn[n - 1];
        u64 rhat = num - qhat * vn[n - 1];
        while (qhat >= base || qhat * vn[n - 2] > ((rhat << 32) | un[j + n - 2])) {
            qhat--;
            rhat += vn[n - 1];
            if (rhat >= base) break;
        }
        int64_t k = 0, t;
        for (int i = 0; i < n; i++) {
            u64 p = qhat * vn[i];
            t = (int64_t)un[i + j] - k - (int64_t)(p & 0xFFFFFFFFu);
            un[i + j] = (u32)t;
            k = (int64_t)(p >> 32) - (t >> 32);
        }
        t = (int64_t)un[j + n] - k;
        un[j + n] = (u32)t;
        qq.w[j] = (u32)qhat;
        if (t < 0) {
            qq.w[j]--;
            u64 c = 0;
            for (int i = 0; i < n; i++) {
                u64 s2 = (u64)un[i + j] + vn[i] + c;
                un[i + j] = (u32)s2;
                c = s2 >> 32;
            }
            un[j + n] += (u32)c;
        }
    }
    qq.n = m - n + 1;
    bn_norm(&qq);
    bn rr;
    rr.n = n;
    for (int i = 0; i < n - 1; i++)
        rr.w[i] = (un[i] >> s) | (s ? (u32)((u64)un[i + 1] << (32 - s)) : 0);
    rr.w[n - 1] = un[n - 1] >> s;
    bn_norm(&rr);
    *q = qq;
    *r = rr;
}

/* ------------------------------------------------------------------ */
/* Chinese remaindering                                                 */
/* ------------------------------------------------------------------ */
#define MAXB 24
typedef struct {
    int n;
    u64 m[MAXB];
    bn M, half;        /* product, floor(product/2) */
    bn hat[MAXB];      /* M / m_i */
    u64 hat_inv[MAXB]; /* (M / m_i)^-1 mod m_i */
} crt_basis;

static void crt_init(crt_basis *B, const u64 *m, int n)
{
    B->n = n;
    bn_set_u64(&B->M, 1);
    for (int i = 0; i < n; i++) {
        B->m[i] = m[i];
        bn t;
        bn_mul_u64(&t, &B->M, m[i]);
        B->M = t;
    }
    B->half = B->M;
    bn_shr1(&B->half);
    for (int i = 0; i < n; i++) {
        bn_set_u64(&B->hat[i], 1);
        for (int j = 0; j < n; j++)
            if (j != i) {
                bn t;
                bn_mul_u64(&t, &B->hat[i], m[j]);
                B->hat[i] = t;
            }
        B->hat_inv[i] = invmod_prime(bn_mod_u64(&B->hat[i], m[i]), m[i]);
    }
}
/* x in [0, M) with x = res[i] mod m_i:  x = sum_i ((res_i * hat_inv_i) mod m_i) * hat_i  mod M */
static void crt_lift(const crt_basis *B, const u64 *res, bn *x)
{
    bn acc;
    acc.n = 0;
    for (int i = 0; i < B->n; i++) {
        u64 c = mulmod(res[i] % B->m[i], B->hat_inv[i], B->m[i]);
        bn t, s;
        bn_mul_u64(&t, &B->hat[i], c);
        bn_add(&s, &acc, &t);
        acc = s;
    }
    while (bn_cmp(&acc, &B->M) >= 0) {
        bn s;
        bn_sub(&s, &acc, &B->M);
        acc = s;
    }
    *x = acc;
}
/* centred lift: magnitude and sign of the representative in (-M/2, M/2] */
static void crt_lift_centred(const crt_basis *B, const u64 *res, bn *mag, int *neg)
{
    bn x;
    crt_lift(B, res, &x);
    if (bn_cmp(&x, &B->half) > 0) {
        bn_sub(mag, &B->M, &x);
        *neg = 1;
    } else {
        *mag = x;
        *neg = 0;
    }
}
static u64 signed_mod(const bn *mag, int neg, u64 m)
{
    u64 r = bn_mod_u64(mag, m);
    return (neg && r) ? m - r : r;
}

/* ------------------------------------------------------------------ */
/* context                                                              */
/* ------------------------------------------------------------------ */
#define MAXP 16
typedef struct orc_ctx {
    int log2n, N, k, nsp, alpha, dnum;
    u64 t;
    u64 q[MAXP], p[MAXP], qp[2 * MAXP];
    u64 psi_qp[2 * MAXP];   /* a primitive 2N-th root for each of q.., p.. */
    crt_basis cQ, cP, cPQ;
    crt_basis cDig[MAXP];   /* one basis per key-switch digit */
    /* private basis for integer polynomial products */
    crt_basis cM;
    u64 psi_m[MAXB];
} orc_ctx;

orc_ctx *orc_create(int log2n, int k, const u64 *q, int nsp, const u64 *p, u64 t, int alpha)
{
    if (k < 1 || k > MAXP || nsp < 1 || nsp > MAXP || alpha < 1 || k % alpha) return NULL;
    orc_ctx *c = (orc_ctx *)calloc(1, sizeof(orc_ctx));
    c->log2n = log2n;
    c->N = 1 << log2n;
    c->k = k;
    c->nsp = nsp;
    c->alpha = alpha;
    c->dnum = k / alpha;
    c->t = t;
    u64 two_n = 2 * (u64)c->N;
    for (int i = 0; i < k; i++) {
        if (!is_prime_u64(q[i]) || q[i] % two_n != 1) { free(c); return NULL; }
        c->q[i] = c->qp[i] = q[i];
    }
    for (int i = 0; i < nsp; i++) {
        if (!is_prime_u64(p[i]) || p[i] % two_n != 1) { free(c); return NULL; }
        c->p[i] = c->qp[k + i] = p[i];
    }
    for (int i = 0; i < k + nsp; i++) c->psi_qp[i] = orc_min_psi(c->N, c->qp[i]);
    crt_init(&c->cQ, c->q, k);
    crt_init(&c->cP, c->p, nsp);
    crt_init(&c->cPQ, c->qp, k + nsp);
    for (int j = 0; j < c->dnum; j++) crt_init(&c->cDig[j], c->q + j * alpha, alpha);
    /* integer products of two centred elements have |coeff| <= N * (Q/2)^2 * 2;
     * take private primes until their product exceeds 8 * N * Q^2. */
    bn bound, tmp;
    bn_mul(&bound, &c->cQ.M, &c->cQ.M);
    bn_mul_u64(&tmp, &bound, 8 * (u64)c->N);
    bound = tmp;
    u64 mlist[MAXB];
    int nm = 0;
    bn prod;
    bn_set_u64(&prod, 1);
    u64 step = (u64)1 << 18; /* m = 1 mod 2^18 supports N up to 2^17 */
    u64 cand = (((u64)1 << 61) / step) * step + 1;
    while (bn_cmp(&prod, &bound) <= 0 && nm < MAXB) {
        cand -= step;
        if (!is_prime_u64(cand)) continue;
        mlist[nm++] = cand;
        bn_mul_u64(&tmp, &prod, cand);
        prod = tmp;
    }
    crt_init(&c->cM, mlist, nm);
    for (int i = 0; i < nm; i++) c->psi_m[i] = orc_min_psi(c->N, mlist[i]);
    return c;
}
void orc_destroy(orc_ctx *c) { free(c); }
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ */
/* evaluator operations                                                 */
/* ------------------------------------------------------------------ */

/* out = a + b, ncomp components */
void orc_add(const orc_ctx *c, const u64 *a, const u64 *b, u64 *out, int ncomp)
{
    int N = c->N, k = c->k;
    for (int cc = 0; cc < ncomp; cc++)
        for (int i = 0; i < k; i++)
            for (int n = 0; n < N; n++) {
                size_t o = ((size_t)cc * k + i) * N + n;
                out[o] = addmod(a[o], b[o], c->q[i]);
            }
}

/* prod_c += (a (x) b)_c over Z, in the private basis (prod = uint64[3][nm][N]):
 * e0 = a0 b0, e1 = a0 b1 + a1 b0, e2 = a1 b1, every operand lifted to its centred representative */
static void add_tensor(const orc_ctx *c, const u64 *a2, const u64 *b2, u64 *prod)
{
    const int N = c->N, k = c->k, nm = c->cM.n;
    const u64 *polys[4] = {a2, a2 + (size_t)k * N, b2, b2 + (size_t)k * N};
    u64 *lift = (u64 *)malloc(sizeof(u64) * (size_t)4 * nm * N);
    /* centred integer lift of every coefficient, reduced into the private basis */
#pragma omp parallel for collapse(2) schedule(static)
    for (int pi = 0; pi < 4; pi++)
        for (int n = 0; n < N; n++) {
            u64 res[MAXP];
            for (int i = 0; i < k; i++) res[i] = polys[pi][(size_t)i * N + n];
            bn mag;
            int neg;
            crt_lift_centred(&c->cQ, res, &mag, &neg);
            for (int j = 0; j < nm; j++)
                lift[((size_t)pi * nm + j) * N + n] = signed_mod(&mag, neg, c->cM.m[j]);
        }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < nm; j++) {
        u64 m = c->cM.m[j], psi = c->psi_m[j];
        const u64 *a0 = lift + ((size_t)0 * nm + j) * N, *a1 = lift + ((size_t)1 * nm + j) * N;
        const u64 *b0 = lift + ((size_t)2 * nm + j) * N, *b1 = lift + ((size_t)3 * nm + j) * N;
        u64 *e[3] = {prod + ((size_t)0 * nm + j) * N, prod + ((size_t)1 * nm + j) * N, prod + ((size_t)2 * nm + j) * N};
        u64 *tmp = (u64 *)malloc(sizeof(u64) * (size_t)N);
        polymul_psi(a0, b0, tmp, N, m, psi);
        for (int n = 0; n < N; n++) e[0][n] = addmod(e[0][n], tmp[n], m);
        polymul_psi(a0, b1, tmp, N, m, psi);
        for (int n = 0; n < N; n++) e[1][n] = addmod(e[1][n], tmp[n], m);
        polymul_psi(a1, b0, tmp, N, m, psi);
        for (int n = 0; n < N; n++) e[1][n] = addmod(e[1][n], tmp[n], m);
        polymul_psi(a1, b1, tmp, N, m, psi);
        for (int n = 0; n < N; n++) e[2][n] = addmod(e[2][n], tmp[n], m);
        free(tmp);
    }
    free(lift);
}

/* d = round(t * e / Q) mod Q, exactly, for the three components held in the private basis */
static void scale_tensor(const orc_ctx *c, const u64 *prod, u64 *out3)
{
    const int N = c->N, k = c->k, nm = c->cM.n;
    bn twoQ = c->cQ.M;
    bn_shl1(&twoQ);
#pragma omp parallel for collapse(2) schedule(static)
    for (int cc = 0; cc < 3; cc++)
        for (int n = 0; n < N; n++) {
            u64 res[MAXB];
            for (int j = 0; j < nm; j++) res[j] = prod[((size_t)cc * nm + j) * N + n];
            bn mag, num, tmp, quo, rem;
            int neg;
            crt_lift_centred(&c->cM, res, &mag, &neg);
            bn_mul_u64(&num, &mag, 2 * c->t);      /* 2 t |e| */
            bn_add(&tmp, &num, &c->cQ.M);          /* + Q */
            bn_divmod(&quo, &rem, &tmp, &twoQ);    /* floor((2t|e| + Q) / 2Q) = round(t|e|/Q) */
            for (int i = 0; i < k; i++)
                out3[((size_t)cc * k + i) * N + n] = signed_mod(&quo, neg, c->q[i]);
        }
}

/* BFV multiplication without relinearisation: out3 = round(t/Q * (a (x) b)) mod Q */
void orc_mul(const orc_ctx *c, const u64 *a2, const u64 *b2, u64 *out3)
{
    u64 *prod = (u64 *)calloc((size_t)3 * c->cM.n * c->N, sizeof(u64));
    add_tensor(c, a2, b2, prod);
    scale_tensor(c, prod, out3);
    free(prod);
}

/* Sum of n products with ONE scaling: out3 = round(t/Q * sum_u (a_u (x) b_u)) mod Q, the tensor
 * products summed over Z before the rounding division (a2s, b2s: n ciphertexts back to back).
 * It decrypts to the sum of the n slot-wise products like the sum of n separately scaled ones, from
 * which it differs by less than n/2 + 1 per coefficient (one rounding instead of n).  Returns
 * nonzero when the private basis cannot hold the sum (n N Q^2 must stay below its modulus). */
int orc_mul_sum(const orc_ctx *c, const u64 *a2s, const u64 *b2s, int n, u64 *out3)
{
    const size_t ct = (size_t)2 * c->k * c->N;
    bn need, tmp;
    bn_mul(&tmp, &c->cQ.M, &c->cQ.M);
    bn_mul_u64(&need, &tmp, (u64)c->N * (u64)(n > 0 ? n : 1));
    if (n < 1 || bn_cmp(&need, &c->cM.M) >= 0) return 1;
    u64 *prod = (u64 *)calloc((size_t)3 * c->cM.n * c->N, sizeof(u64));
    for (int u = 0; u < n; u++) add_tensor(c, a2s + u * ct, b2s + u * ct, prod);
    scale_tensor(c, prod, out3);
    free(prod);
    return 0;
}

/* acc_c += sum_j digit_j * ksk_{j,c} in Z_{PQ}[X]/(X^N+1), residue by residue
 * (dig = uint64[dnum][k+nsp][N], acc = uint64[2][k+nsp][N]) */
static void add_digit_products(const orc_ctx *c, const u64 *dig, const u64 *ksk, u64 *acc)
{
    const int N = c->N, k = c->k, nsp = c->nsp, L = k + nsp, dnum = c->dnum;
#pragma omp parallel for collapse(2) schedule(static)
    for (int cc = 0; cc < 2; cc++)
        for (int r = 0; r < L; r++) {
            u64 m = c->qp[r];
            u64 *tmp = (u64 *)malloc(sizeof(u64) * (size_t)N);
            u64 *dst = acc + ((size_t)cc * L + r) * N;
            for (int j = 0; j < dnum; j++) {
                const u64 *key = ksk + (((size_t)j * 2 + cc) * L + r) * N;
                polymul_psi(dig + ((size_t)j * L + r) * N, key, tmp, N, m, c->psi_qp[r]);
                for (int n = 0; n < N; n++) dst[n] = addmod(dst[n], tmp[n], m);
            }
            free(tmp);
        }
}

/* u_c = floor((A_c + floor(P/2)) / P) mod Q with A_c, given by its residues, taken in [0, PQ);
 * acc = uint64[2][k+nsp][N], u2 = uint64[2][k][N] */
static void divide_by_special(const orc_ctx *c, const u64 *acc, u64 *u2)
{
    const int N = c->N, k = c->k, L = k + c->nsp;
#pragma omp parallel for collapse(2) schedule(static)
    for (int cc = 0; cc < 2; cc++)
        for (int n = 0; n < N; n++) {
            u64 res[2 * MAXP];
            for (int r = 0; r < L; r++) res[r] = acc[((size_t)cc * L + r) * N + n];
            bn A, s, quo, rem;
            crt_lift(&c->cPQ, res, &A);
            bn_add(&s, &A, &c->cP.half);
            bn_divmod(&quo, &rem, &s, &c->cP.M);
            for (int i = 0; i < k; i++)
                u2[((size_t)cc * k + i) * N + n] = bn_mod_u64(&quo, c->q[i]);
        }
}

/* Second half of a key switch, from the digits already reduced modulo every prime of P*Q:
 * A_c = sum_j digit_j * ksk_{j,c}, u_c = round(A_c / P) mod Q as above */
static void switch_digits(const orc_ctx *c, const u64 *dig, const u64 *ksk, u64 *u2)
{
    u64 *acc = (u64 *)calloc((size_t)2 * (c->k + c->nsp) * c->N, sizeof(u64));
    add_digit_products(c, dig, ksk, acc);
    divide_by_special(c, acc, u2);
    free(acc);
}

/* hybrid key switch of one ring element d (uint64[k][N]) with key ksk; u2 = uint64[2][k][N] */
void orc_keyswitch(const orc_ctx *c, const u64 *d, const u64 *ksk, u64 *u2)
{
    const int N = c->N, k = c->k, nsp = c->nsp, L = k + nsp, dnum = c->dnum, alpha = c->alpha;
    u64 *dig = (u64 *)malloc(sizeof(u64) * (size_t)dnum * L * N);
    /* digit j = d mod Q_j as the integer in [0, Q_j), reduced modulo every prime of P*Q */
#pragma omp parallel for collapse(2) schedule(static)
    for (int j = 0; j < dnum; j++)
        for (int n = 0; n < N; n++) {
            u64 res[MAXP];
            for (int a = 0; a < alpha; a++) res[a] = d[(size_t)(j * alpha + a) * N + n];
            bn x;
            crt_lift(&c->cDig[j], res, &x);
            for (int r = 0; r < L; r++) dig[((size_t)j * L + r) * N + n] = bn_mod_u64(&x, c->qp[r]);
        }
    switch_digits(c, dig, ksk, u2);
    free(dig);
}

/* (d0, d1, d2) -> (d0 + u0, d1 + u1), u = keyswitch(d2, rlk) */
void orc_relin(const orc_ctx *c, const u64 *in3, const u64 *rlk, u64 *out2)
{
    const size_t comp = (size_t)c->k * c->N;
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * comp);
    orc_keyswitch(c, in3 + 2 * comp, rlk, u);
    orc_add(c, in3, u, out2, 2);
    free(u);
}

/* Galois map on one ring element: the coefficient at index i goes to index
 * i*g mod N, negated when i*g mod 2N >= N. g odd, 0 < g < 2N. */
void orc_galois_poly(const orc_ctx *c, const u64 *in, u64 g, u64 *out)
{
    const int N = c->N, k = c->k;
    for (int i = 0; i < k; i++)
        for (int n = 0; n < N; n++) {
            u64 e = ((u64)n * g) % (2 * (u64)N);
            u64 v = in[(size_t)i * N + n];
            if (e >= (u64)N) out[(size_t)i * N + (e - N)] = v ? c->q[i] - v : 0;
            else out[(size_t)i * N + e] = v;
        }
}

/* out = (sigma_g(c0) + u0, u1), u = keyswitch(sigma_g(c1), gk) */
void orc_rotate(const orc_ctx *c, const u64 *in2, u64 g, const u64 *gk, u64 *out2)
{
    const size_t comp = (size_t)c->k * c->N;
    u64 *s = (u64 *)malloc(sizeof(u64) * 2 * comp);
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * comp);
    orc_galois_poly(c, in2, g, s);
    orc_galois_poly(c, in2 + comp, g, s + comp);
    orc_keyswitch(c, s + comp, gk, u);
    for (int i = 0; i < c->k; i++)
        for (int n = 0; n < c->N; n++) {
            size_t o = (size_t)i * c->N + n;
            out2[o] = addmod(s[o], u[o], c->q[i]);
            out2[comp + o] = u[comp + o];
        }
    free(s);
    free(u);
}

/* digit_j of the ring element d (uint64[k][N]) as integer polynomials, mapped by sigma_g over the
 * integers (index i -> i*g mod N, negated when i*g mod 2N >= N) and then reduced modulo every
 * prime of P*Q: dig = uint64[dnum][k+nsp][N] */
static void galois_of_digits(const orc_ctx *c, const u64 *d, u64 g, u64 *dig)
{
    const int N = c->N, L = c->k + c->nsp, dnum = c->dnum, alpha = c->alpha;
#pragma omp parallel for collapse(2) schedule(static)
    for (int j = 0; j < dnum; j++)
        for (int n = 0; n < N; n++) {
            u64 res[MAXP];
            for (int a = 0; a < alpha; a++) res[a] = d[(size_t)(j * alpha + a) * N + n];
            bn x;
            crt_lift(&c->cDig[j], res, &x);
            const u64 e = ((u64)n * g) % (2 * (u64)N);
            const int neg = e >= (u64)N;
            const size_t dst = (size_t)(neg ? e - N : e);
            for (int r = 0; r < L; r++) {
                const u64 v = bn_mod_u64(&x, c->qp[r]);
                dig[((size_t)j * L + r) * N + dst] = (neg && v) ? c->qp[r] - v : v;
            }
        }
}

/* Hoisted rotation: the digits are taken from c1 as it stands -- digit_j = c1 mod Q_j as the
 * integer polynomial with coefficients in [0, Q_j), the same for every Galois element applied to
 * this ciphertext -- and the Galois map acts on those integer polynomials: the coefficient x at
 * index i goes to index i*g mod N as +x or, when i*g mod 2N >= N, as the negative integer -x.
 *   u = second half of the key switch on (sigma_g(digit_j))_j with gk;  out = (sigma_g(c0) + u0, u1).
 * Differs from orc_rotate in where the lift happens (there sigma_g(c1) mod Q_j is lifted to
 * [0, Q_j), i.e. a negated coefficient becomes Q_j - x): the results decrypt to the same slots but
 * are different ciphertexts. */
void orc_rotate_hoisted(const orc_ctx *c, const u64 *in2, u64 g, const u64 *gk, u64 *out2)
{
    const int N = c->N, k = c->k, L = k + c->nsp, dnum = c->dnum;
    const size_t comp = (size_t)k * N;
    u64 *dig = (u64 *)malloc(sizeof(u64) * (size_t)dnum * L * N);
    u64 *s0 = (u64 *)malloc(sizeof(u64) * comp);
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * comp);
    galois_of_digits(c, in2 + comp, g, dig);
    switch_digits(c, dig, gk, u);
    orc_galois_poly(c, in2, g, s0);
    for (int i = 0; i < k; i++)
        for (int n = 0; n < N; n++) {
            size_t o = (size_t)i * N + n;
            out2[o] = addmod(s0[o], u[o], c->q[i]);
            out2[comp + o] = u[comp + o];
        }
    free(dig);
    free(s0);
    free(u);
}

/* Sum of a ciphertext and a series of its hoisted rotations with ONE division by P:
 *   A_c = sum_i sum_j sigma_{g_i}(digit_j) * gk_i[j][c]  in Z_{PQ}[X]/(X^N+1),  digits of c1 as in
 *   orc_rotate_hoisted;  u_c = floor((A_c + floor(P/2)) / P) mod Q;
 *   out = (c0 + sum_i sigma_{g_i}(c0) + u0,  c1 + u1).
 * Rounding A_c / P is additive up to the rounding itself, so u differs from the sum of the n_rot
 * separately rounded key-switch outputs by less than n_rot per coefficient: the result decrypts to
 * the slot-wise sum x + sum_i rotate(x, g_i) with one rounding error instead of n_rot, and is a
 * different ciphertext from the sum of n_rot separately rotated ones.  gks = n_rot key pointers. */
void orc_rotate_sum_hoisted(const orc_ctx *c, const u64 *in2, int n_rot, const u64 *gs, const u64 *const *gks,
                            u64 *out2)
{
    const int N = c->N, k = c->k, L = k + c->nsp, dnum = c->dnum;
    const size_t comp = (size_t)k * N;
    u64 *dig = (u64 *)malloc(sizeof(u64) * (size_t)dnum * L * N);
    u64 *acc = (u64 *)calloc((size_t)2 * L * N, sizeof(u64));
    u64 *s0 = (u64 *)malloc(sizeof(u64) * comp);
    u64 *u = (u64 *)malloc(sizeof(u64) * 2 * comp);
    memcpy(out2, in2, sizeof(u64) * 2 * comp);
    for (int i = 0; i < n_rot; i++) {
        galois_of_digits(c, in2 + comp, gs[i], dig);
        add_digit_products(c, dig, gks[i], acc);
        orc_galois_poly(c, in2, gs[i], s0);
        for (int r = 0; r < k; r++)
            for (int n = 0; n < N; n++) {
                size_t o = (size_t)r * N + n;
                out2[o] = addmod(out2[o], s0[o], c->q[r]);
            }
    }
    divide_by_special(c, acc, u);
    for (int r = 0; r < k; r++)
        for (int n = 0; n < N; n++) {
            size_t o = (size_t)r * N + n;
            out2[o] = addmod(out2[o], u[o], c->q[r]);
            out2[comp + o] = addmod(out2[comp + o], u[comp + o], c->q[r]);
        }
    free(dig);
    free(acc);
    free(s0);
    free(u);
}

/* ciphertext times plaintext polynomial pt (uint64[N], coefficients in [0,t)),
 * the plaintext lifted to its centred representative in (-t/2, t/2] */
void orc_mul_plain(const orc_ctx *c, const u64 *in2, const u64 *pt, u64 *out2)
{
    const int N = c->N, k = c->k;
    u64 *lifted = (u64 *)malloc(sizeof(u64) * (size_t)N);
    for (int i = 0; i < k; i++) {
        u64 m = c->q[i];
        for (int n = 0; n < N; n++) {
            u64 v = pt[n] % c->t;
            lifted[n] = (v > (c->t - 1) / 2) ? m - (c->t - v) : v;
        }
        for (int cc = 0; cc < 2; cc++)
            polymul_psi(in2 + ((size_t)cc * k + i) * N, lifted, out2 + ((size_t)cc * k + i) * N, N, m,
                        c->psi_qp[i]);
    }
    free(lifted);
}

/* ciphertext +- plaintext: (c0 +- floor(Q/t) * pt, c1), pt coefficients in [0,t); the quotient
 * floor(Q/t) is taken over the integers (long division of Q by t) and then reduced modulo each q_i */
void orc_add_plain(const orc_ctx *c, const u64 *in2, const u64 *pt, int negative, u64 *out2)
{
    const int N = c->N, k = c->k;
    bn tt, delta, rem;
    tt.n = 1; tt.w[0] = (u32)c->t; bn_norm(&tt);
    if (c->t >> 32) { tt.n = 2; tt.w[1] = (u32)(c->t >> 32); }
    bn_divmod(&delta, &rem, &c->cQ.M, &tt);
    for (int i = 0; i < k; i++) {
        const u64 m = c->q[i], d = bn_mod_u64(&delta, m);
        for (int n = 0; n < N; n++) {
            const size_t o = (size_t)i * N + n;
            const u64 x = mulmod(d, pt[n] % c->t, m);
            out2[o] = negative ? submod(in2[o], x, m) : addmod(in2[o], x, m);
            out2[(size_t)k * N + o] = in2[(size_t)k * N + o];
        }
    }
}

/* ------------------------------------------------------------------ */
/* hooks used only by the pin tests and the host-side client            */
/* ------------------------------------------------------------------ */

/* x = the integer in [0, prod m_i) with the given residues; little-endian 32-bit words */
int orc_test_crt(const u64 *m, int n, const u64 *res, u32 *words, int cap)
{
    crt_basis *B = (crt_basis *)malloc(sizeof(crt_basis));
    bn x;
    crt_init(B, m, n);
    crt_lift(B, res, &x);
    free(B);
    if (x.n > cap) return -1;
    memcpy(words, x.w, sizeof(u32) * (size_t)x.n);
    return x.n;
}
/* quotient and remainder of two big integers given as little-endian 32-bit words */
int orc_test_divmod(const u32 *a, int an, const u32 *b, int bn_, u32 *q, int *qn, u32 *r, int *rn)
{
    bn A, B, Qo, R;
    if (an > BN_CAP - 2 || bn_ > BN_CAP - 2 || bn_ == 0) return -1;
    A.n = an; memcpy(A.w, a, sizeof(u32) * (size_t)an); bn_norm(&A);
    B.n = bn_; memcpy(B.w, b, sizeof(u32) * (size_t)bn_); bn_norm(&B);
    if (B.n == 0) return -1;
    bn_divmod(&Qo, &R, &A, &B);
    *qn = Qo.n; memcpy(q, Qo.w, sizeof(u32) * (size_t)Qo.n);
    *rn = R.n; memcpy(r, R.w, sizeof(u32) * (size_t)R.n);
    return 0;
}
int orc_test_is_prime(u64 n) { return is_prime_u64(n); }
int orc_private_basis(const orc_ctx *c, u64 *m, int cap)
{
    if (c->cM.n > cap) return -1;
    for (int i = 0; i < c->cM.n; i++) m[i] = c->cM.m[i];
    return c->cM.n;
}
