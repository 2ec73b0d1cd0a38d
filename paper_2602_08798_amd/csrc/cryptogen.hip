// C ABI of the library (see include/cryptogen.h): context set-up on the host,
// argument checks, and the launch sequences of the evaluator operations.
#include "../../include/cryptogen.h"
#include "../../include/cryptogen_bench.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <tuple>
#include <unordered_map>
#include <vector>

#include "kernels.hpp"

using namespace cg;

typedef unsigned __int128 u128;

// Workspace of cg_mul_relin_static, the entry point for callers that cannot allocate: device
// memory that belongs to the loaded library itself (one copy per GPU, held until the process
// ends).  In host code this name is only a handle for the runtime's symbol look-up; the address the
// kernels get is the one hipGetSymbolAddress returns on the device in question, kept below.
__device__ __align__(256) unsigned char scratch[CG_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];   // per device; null until a context was created there
// the array's address on `device`, which must be the current device
static int static_scratch_address(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return CG_EINVAL;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CG_EHIP;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return CG_OK;
}

// ---------------------------------------------------------------------------
// host integer helpers (set-up only)
// ---------------------------------------------------------------------------
static uint64_t h_mul(uint64_t a, uint64_t b, uint64_t m) { return (uint64_t)((u128)a * b % m); }
static uint64_t h_pow(uint64_t a, uint64_t e, uint64_t m)
{
    uint64_t r = 1;
    a %= m;
    for (; e; e >>= 1, a = h_mul(a, a, m))
        if (e & 1) r = h_mul(r, a, m);
    return r;
}
static uint64_t h_inv(uint64_t a, uint64_t m) { return h_pow(a % m, m - 2, m); }
// Primality below 2^64 by strong-probable-prime tests to the seven bases of Sinclair's set, which
// has no composite below 2^64 passing all of them; trial division first, to leave early.
static bool h_is_prime(uint64_t n)
{
    if (n < 4) return n == 2 || n == 3;
    if (!(n & 1)) return false;
    for (uint64_t f = 3; f < 64; f += 2) {
        if (n == f) return true;
        if (n % f == 0) return false;
    }
    const int two = __builtin_ctzll(n - 1);
    const uint64_t odd = (n - 1) >> two;
    static const uint64_t bases[7] = {2, 325, 9375, 28178, 450775, 9780504, 1795265022};
    for (uint64_t b : bases) {
        uint64_t y = h_pow(b % n, odd, n);
        if (y <= 1 || y == n - 1) continue;            // b = 0 mod n gives y = 0: no witness
        int sq = 1;
        while (sq < two && y != n - 1) { y = h_mul(y, y, n); sq++; }
        if (y != n - 1) return false;
    }
    return true;
}
// smallest primitive 2N-th root of unity mod p (the convention of cg_ntt_forward): any primitive
// root, then the minimum over its N odd powers, which are all the primitive 2N-th roots
static uint64_t h_min_root(uint64_t p, uint64_t n)
{
    const uint64_t cof = (p - 1) / (2 * n);
    uint64_t any = 0;
    for (uint64_t cand = 2; !any; cand++) {
        const uint64_t r = h_pow(cand, cof, p);      // order divides 2N; it is 2N iff r^N = -1
        if (h_pow(r, n, p) == p - 1) any = r;
    }
    const uint64_t step = h_mul(any, any, p);
    uint64_t lo = any, w = any;
    for (uint64_t i = 1; i < n; i++) {
        w = h_mul(w, step, p);
        lo = w < lo ? w : lo;
    }
    return lo;
}
static uint32_t h_bitrev(uint32_t x, int bits)
{
    uint32_t r = 0;
    for (int i = 0; i < bits; i++) { r = (r << 1) | (x & 1); x >>= 1; }
    return r;
}
static double h_centred(uint64_t x, uint64_t p) { return x > p / 2 ? -(double)(p - x) : (double)x; }

// ---------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------
struct cg_ctx {
    int logn, N, k, nsp, alpha, dnum, l, L, KL, np;
    uint64_t t;
    uint64_t pr[MAXPR];
    DevConst hc;
    DevConst *dc;
    double *tw, *itw;     // [np][N] forward / inverse twiddles (centred doubles, bit-reversed order)
    uint32_t *tab;        // scratch prime-index table for the public transform entry points
    uint32_t tab_cap;
    int device, n_cu;
    void *static_ws;      // this device's copy of the library-owned scratch array
    // resident workgroups per compute unit of every transform-kernel instantiation this context
    // launches, keyed by the kernel's address: filled by cg_create (a dry pass over all launch
    // sequences), so that no launch has to ask the runtime; the lock covers a late first use
    std::mutex *occ_mu;
    std::unordered_map<const void *, int> *occ;
    bool dry;             // set-up pass: launches compute their grid and return without launching
    int elems, elems_fwd; // elements per thread in the inverse / forward transform kernels (8 or 16)
    // workspace limbs (N * 8 bytes) per unit
    int ws_total;
    // two side streams (default priority) and fork/join events for entry points that run
    // independent branches side by side
    hipStream_t side[2];
    hipEvent_t ev_fork, ev_join[2];
    // optional per-launch timing with HIP events (benchmark support)
    bool prof_on;
    uint32_t prof_n, prof_cap;
    hipEvent_t *prof_ev;      // 2 * prof_cap events
    uint8_t *prof_id;
    double *prof_bytes;
    double *prof_items;
};

// kernel classes for the timing facility
enum KernelId {
    KID_FWD_MULQ = 0, KID_FWD_MULB, KID_FWD_MODUP, KID_FWD_ROWS, KID_FWD_PLAIN,
    KID_INV_TENSOR, KID_INV_U64, KID_INV_MULPLAIN, KID_SCALE, KID_INV_KSINNER, KID_MODDOWN,
    KID_ADD, KID_SUM_GROUPS, KID_INV_KSSUM, KID_MODDOWN_SUM, KID_INV_TENSORSUM, KID_COUNT
};
static const char *const kKernelNames[KID_COUNT] = {
    "ntt_fwd<mul,q-rows>", "ntt_fwd<mul,aux-rows>", "ntt_fwd<modup>", "ntt_fwd<rows>",
    "ntt_fwd<plain>", "ntt_inv<tensor>", "ntt_inv<u64>", "ntt_inv<mul_plain>", "scale",
    "ntt_inv<ks_inner>", "moddown", "add", "sum_groups", "ntt_inv<ks_sum>", "moddown<sum>",
    "ntt_inv<tensor_sum>"};

// Brackets one launch with two events when profiling is on.
struct ProfScope {
    cg_ctx *c;
    hipStream_t s;
    int slot;
    // items: residue rows a transform launch works through, batch units for a pointwise launch
    ProfScope(cg_ctx *c_, hipStream_t s_, int id, double bytes, double items) : c(c_), s(s_), slot(-1)
    {
        if (c->prof_on && c->prof_n < c->prof_cap) {
            slot = (int)c->prof_n++;
            c->prof_id[slot] = (uint8_t)id;
            c->prof_bytes[slot] = bytes;
            c->prof_items[slot] = items;
            (void)hipEventRecord(c->prof_ev[2 * slot], s);
        }
    }
    ~ProfScope()
    {
        if (slot >= 0) (void)hipEventRecord(c->prof_ev[2 * slot + 1], s);
    }
};

static void fill_conv(ConvTab &T, const uint64_t *pr, const int *sidx, int ns, const int *tidx, int nt)
{
    memset(&T, 0, sizeof(T));
    T.ns = ns;
    T.nt = nt;
    for (int i = 0; i < ns; i++) T.sidx[i] = sidx[i];
    for (int j = 0; j < nt; j++) T.tidx[j] = tidx[j];
    for (int i = 0; i < ns; i++)
        for (int j = i + 1; j < ns; j++) {
            const uint64_t si = pr[sidx[i]], sj = pr[sidx[j]];
            T.inv[i][j] = h_centred(h_inv(si % sj, sj), sj);
        }
    // digits of floor(S/2): its residue modulo s_i is (s_i - 1)/2 because S = 0 and 2 is invertible
    uint64_t a[MAXS];
    for (int j = 0; j < ns; j++) {
        const uint64_t sj = pr[sidx[j]];
        uint64_t v = (sj - 1) / 2;
        for (int i = 0; i < j; i++) {
            const uint64_t si = pr[sidx[i]];
            v = h_mul((v + sj - a[i] % sj) % sj, h_inv(si % sj, sj), sj);
        }
        a[j] = v;
        T.half[j] = (double)v;
    }
    for (int j = 0; j < nt; j++) {
        const uint64_t tj = pr[tidx[j]];
        uint64_t prod = 1;
        for (int i = 0; i < ns; i++) {
            T.s_mod_t[i][j] = h_centred(pr[sidx[i]] % tj, tj);
            prod = h_mul(prod, pr[sidx[i]] % tj, tj);
        }
        T.S_mod_t[j] = h_centred(prod, tj);
    }
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
#define CG_REQUIRE(cond) do { if (!(cond)) return CG_EINVAL; } while (0)
#define CG_HIP(call) do { if ((call) != hipSuccess) return CG_EHIP; } while (0)
// Launch through the runtime's C entry point: its return value is this launch's own status, so an
// error that other code left pending in the thread is neither reported as ours nor cleared.
template <class... P, class... A>
static int launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t s, A... args)
{
    std::tuple<P...> pack{static_cast<P>(args)...};
    void *ptrs[sizeof...(P)];
    int i = 0;
    std::apply([&](auto &...e) { ((ptrs[i++] = static_cast<void *>(&e)), ...); }, pack);
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, 0, s) == hipSuccess ? CG_OK
                                                                                                         : CG_EHIP;
}

extern "C" const char *cg_strerror(int status)
{
    switch (status) {
    case CG_OK: return "ok";
    case CG_EINVAL: return "invalid argument";
    case CG_ENOMEM: return "out of device memory";
    case CG_EHIP: return "HIP runtime error";
    case CG_ESCRATCH: return "batch needs more scratch than the library's static array holds";
    default: return "unknown status";
    }
}

static int warm_launch_table(cg_ctx *c);

extern "C" int cg_create(cg_ctx **out, const cg_params *prm)
{
    CG_REQUIRE(out && prm && prm->q && prm->p);
    *out = nullptr;
    CG_REQUIRE(prm->log2n >= 12 && prm->log2n <= 14);
    CG_REQUIRE(prm->k >= 1 && prm->k <= 6 && prm->nsp >= 1 && prm->nsp <= 2);
    CG_REQUIRE(prm->alpha >= 1 && prm->alpha <= 3 && prm->k % prm->alpha == 0);
    // a digit of alpha primes against fewer special primes makes P smaller than Q_j by a whole prime:
    // every result would still match its definition, but a key switch would add noise of the size of
    // a prime and silently use up the decryption budget
    CG_REQUIRE(prm->alpha <= prm->nsp);
    CG_REQUIRE((prm->t & 1) && prm->t > 2 && prm->t < (1u << 20));
    const uint64_t N = 1ull << prm->log2n;
    cg_ctx *c = new (std::nothrow) cg_ctx();
    if (!c) return CG_ENOMEM;
    memset(c, 0, sizeof(*c));
    c->occ_mu = new (std::nothrow) std::mutex();
    c->occ = new (std::nothrow) std::unordered_map<const void *, int>();
    if (!c->occ_mu || !c->occ) { cg_destroy(c); return CG_ENOMEM; }
    c->logn = (int)prm->log2n; c->N = (int)N; c->k = (int)prm->k; c->nsp = (int)prm->nsp;
    c->alpha = (int)prm->alpha; c->dnum = c->k / c->alpha; c->t = prm->t;
    c->l = c->k + 1;
    c->elems = c->logn <= 13 ? 8 : 16;              // 1024 threads per row at N >= 8192, 512 at N = 4096
    c->elems_fwd = c->logn == 13 ? 16 : c->elems;   // two 512-thread workgroups per compute unit at N = 8192
    c->L = c->k + c->nsp;
    c->KL = c->k + c->l;
    int np = 0;
    uint64_t lowest = ~0ull;
    auto ok_prime = [&](uint64_t p) {
        if (!(p > (1ull << 40) && p < (1ull << 50) && p % (2 * N) == 1 && h_is_prime(p))) return false;
        for (int i = 0; i < np; i++) if (c->pr[i] == p) return false;
        return true;
    };
    for (uint32_t i = 0; i < prm->k + prm->nsp; i++) {
        const uint64_t p = i < prm->k ? prm->q[i] : prm->p[i - prm->k];
        if (!ok_prime(p) || p == prm->t) { cg_destroy(c); return CG_EINVAL; }
        c->pr[np++] = p;
        if (p < lowest) lowest = p;
    }
    // auxiliary basis for the tensor product: the special primes plus private primes
    // below every given prime, l = k + 1 in total
    uint64_t cand = lowest;
    while (np < c->k + c->l) {
        cand -= 2 * N;
        if (cand <= (1ull << 40)) { cg_destroy(c); return CG_EINVAL; }
        if (ok_prime(cand) && cand != prm->t) c->pr[np++] = cand;
    }
    c->np = np;
    // the scaled product round(t e / Q) is below t N Q in magnitude and must fit the centred
    // range of the auxiliary basis
    double lgQ = 0, lgB = 0;
    for (int i = 0; i < c->k; i++) lgQ += std::log2((double)c->pr[i]);
    for (int j = 0; j < c->l; j++) lgB += std::log2((double)c->pr[c->k + j]);
    if (!(lgB > lgQ + std::log2((double)c->t) + c->logn + 3)) { cg_destroy(c); return CG_EINVAL; }

    DevConst &H = c->hc;
    memset(&H, 0, sizeof(H));
    H.logn = c->logn; H.k = c->k; H.nsp = c->nsp; H.l = c->l; H.alpha = c->alpha; H.dnum = c->dnum;
    H.L = c->L; H.KL = c->KL; H.np = np; H.tmod = (double)c->t;
    std::vector<double> tw((size_t)np * N), itw((size_t)np * N);
    for (int r = 0; r < np; r++) {
        const uint64_t p = c->pr[r];
        H.mod[r].p = (double)p;
        H.mod[r].u = 1.0 / (double)p;
        const uint64_t psi = h_min_root(p, N);
        std::vector<uint64_t> pw(N);
        pw[0] = 1;
        for (uint64_t i = 1; i < N; i++) pw[i] = h_mul(pw[i - 1], psi, p);
        for (uint64_t j = 0; j < N; j++) {
            const uint64_t w = pw[h_bitrev((uint32_t)j, c->logn)];
            tw[(size_t)r * N + j] = h_centred(w, p);
            itw[(size_t)r * N + j] = h_centred(h_inv(w, p), p);
        }
        const uint64_t ninv = h_inv(N % p, p);
        H.ninv[r] = h_centred(ninv, p);
        H.itw1_ninv[r] = h_centred(h_mul(h_inv(pw[h_bitrev(1, c->logn)], p), ninv, p), p);
    }
    int qi[MAXS], bi[MAXS], all[MAXT], sp[MAXS];
    for (int i = 0; i < c->k; i++) qi[i] = i;
    for (int j = 0; j < c->l; j++) bi[j] = c->k + j;
    for (int r = 0; r < c->L; r++) all[r] = r;
    for (int s = 0; s < c->nsp; s++) sp[s] = c->k + s;
    fill_conv(H.q2b, c->pr, qi, c->k, bi, c->l);
    fill_conv(H.b2q, c->pr, bi, c->l, qi, c->k);
    for (int j = 0; j < c->l; j++) {
        const uint64_t b = c->pr[c->k + j];
        uint64_t prod = 1;
        for (int i = 0; i < c->k; i++) prod = h_mul(prod, c->pr[i] % b, b);
        H.Qinv_b[j] = h_centred(h_inv(prod, b), b);
    }
    for (int j = 0; j < c->dnum; j++) fill_conv(H.dig[j], c->pr, qi + j * c->alpha, c->alpha, all, c->L);
    fill_conv(H.p2q, c->pr, sp, c->nsp, qi, c->k);
    for (int r = 0; r < c->L; r++) {
        const uint64_t m = c->pr[r];
        uint64_t P = 1;
        for (int s = 0; s < c->nsp; s++) P = h_mul(P, c->pr[c->k + s] % m, m);
        H.halfP[r] = (double)h_mul((P + m - 1) % m, h_inv(2, m), m);   // (P-1)/2 mod m, P odd
        if (r < c->k) H.Pinv_q[r] = h_centred(h_inv(P, m), m);
    }
    {
        // floor(Q/t) = (Q - (Q mod t)) / t, and Q = 0 modulo q_i: floor(Q/t) = -(Q mod t) t^-1 (mod q_i)
        uint64_t q_mod_t = 1;
        for (int j = 0; j < c->k; j++) q_mod_t = h_mul(q_mod_t, c->pr[j] % c->t, c->t);
        for (int i = 0; i < c->k; i++) {
            const uint64_t m = c->pr[i];
            const uint64_t d = h_mul(m - q_mod_t % m, h_inv(c->t % m, m), m);
            H.delta_q[i] = h_centred(d % m, m);
        }
    }
    // workspace limbs per unit: three ciphertext temporaries (3k + 2k + 2k) plus the larger of the
    // tensor-product and key-switch scratch areas (kept separate for simplicity)
    c->ws_total = 7 * c->k + (4 * c->l + 7 * c->KL) + (c->dnum * c->L + 2 * c->L);

    if (hipGetDevice(&c->device) != hipSuccess ||
        hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess ||
        c->n_cu < 1) {
        cg_destroy(c);
        return CG_EHIP;
    }
    {
        const int src = static_scratch_address(c->device, &c->static_ws);
        if (src != CG_OK) { cg_destroy(c); return src; }
    }
    const size_t tbytes = (size_t)np * N * sizeof(double);
    c->tab_cap = 1u << 16;
    if (hipMalloc(&c->dc, sizeof(DevConst)) != hipSuccess || hipMalloc(&c->tw, tbytes) != hipSuccess ||
        hipMalloc(&c->itw, tbytes) != hipSuccess ||
        hipMalloc(&c->tab, c->tab_cap * sizeof(uint32_t)) != hipSuccess) {
        cg_destroy(c);
        return CG_ENOMEM;
    }
    if (hipMemcpy(c->dc, &H, sizeof(DevConst), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(c->tw, tw.data(), tbytes, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(c->itw, itw.data(), tbytes, hipMemcpyHostToDevice) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        cg_destroy(c);
        return CG_EHIP;
    }
    bool ok = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 2 && ok; i++)
        ok = hipStreamCreateWithFlags(&c->side[i], hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&c->ev_join[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        cg_destroy(c);
        return CG_EHIP;
    }
    // one dry pass over every launch sequence fills the occupancy table
    c->dry = true;
    const int wrc = warm_launch_table(c);
    c->dry = false;
    if (wrc != CG_OK) {
        cg_destroy(c);
        return wrc;
    }
    *out = c;
    return CG_OK;
}

extern "C" int cg_destroy(cg_ctx *c)
{
    if (!c) return CG_OK;
    (void)hipDeviceSynchronize();
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    for (int i = 0; i < 2; i++) {
        if (c->ev_join[i]) (void)hipEventDestroy(c->ev_join[i]);
        if (c->side[i]) (void)hipStreamDestroy(c->side[i]);
    }
    if (c->dc) (void)hipFree(c->dc);
    if (c->tw) (void)hipFree(c->tw);
    if (c->itw) (void)hipFree(c->itw);
    if (c->tab) (void)hipFree(c->tab);
    for (uint32_t i = 0; i < 2 * c->prof_cap; i++) (void)hipEventDestroy(c->prof_ev[i]);
    delete[] c->prof_ev;
    delete[] c->prof_id;
    delete[] c->prof_bytes;
    delete[] c->prof_items;
    delete c->occ;
    delete c->occ_mu;
    delete c;
    return CG_OK;
}

static size_t limb_bytes(const cg_ctx *c) { return (size_t)c->N * 8; }

extern "C" int cg_get_sizes(const cg_ctx *c, cg_sizes *o)
{
    CG_REQUIRE(c && o);
    o->ct2_bytes = 2 * (size_t)c->k * limb_bytes(c);
    o->ct3_bytes = 3 * (size_t)c->k * limb_bytes(c);
    o->ksk_raw_bytes = (size_t)c->dnum * 2 * c->L * limb_bytes(c);
    o->ksk_bytes = o->ksk_raw_bytes;
    o->plain_bytes = (size_t)c->k * limb_bytes(c);
    o->ws_bytes_per_unit = (size_t)c->ws_total * limb_bytes(c);
    o->ct_ext_bytes = 2 * (size_t)c->KL * limb_bytes(c);
    return CG_OK;
}

extern "C" size_t cg_workspace_bytes(const cg_ctx *c, uint32_t batch)
{
    if (!c) return 0;
    return (size_t)c->ws_total * limb_bytes(c) * (batch ? batch : 1);
}

// Workspace carving: composite operations take their persistent buffers first and hand the
// rest to the primitive sequences, which start again from the pointer they are given.
struct Bump {
    char *p;
    size_t limb;
    template <class T> T *take(size_t limbs)
    {
        T *r = reinterpret_cast<T *>(p);
        p += limbs * limb;
        return r;
    }
};
static Bump bump(const cg_ctx *c, void *ws) { return Bump{static_cast<char *>(ws), limb_bytes(c)}; }

// ---------------------------------------------------------------------------
// launch helpers
// ---------------------------------------------------------------------------
// Transform kernels are persistent: the grid is at most the number of workgroups that are
// resident at once (what the runtime reports for this instantiation's registers and LDS), so
// that every workgroup starts immediately and walks over its rows with the next row prefetched.
template <auto KERNEL>
static unsigned ntt_grid(cg_ctx *c, size_t nwg, int threads)
{
    const void *key = reinterpret_cast<const void *>(KERNEL);
    int per_cu = 0;
    {
        std::lock_guard<std::mutex> g(*c->occ_mu);
        auto it = c->occ->find(key);
        if (it != c->occ->end()) per_cu = it->second;
    }
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, KERNEL, threads, 0) != hipSuccess || n < 1) n = 1;
        per_cu = n;
        std::lock_guard<std::mutex> g(*c->occ_mu);
        (*c->occ)[key] = per_cu;
    }
    const size_t resident = (size_t)per_cu * (size_t)c->n_cu;
    return (unsigned)(nwg < resident ? nwg : resident);
}
// elements per thread for this context's transforms
static int ntt_elems(const cg_ctx *c) { return c->elems; }

template <class LD, class ST>
static int launch_fwd(cg_ctx *c, hipStream_t s, size_t nwg, LD ld, ST st, int kid, double bytes)
{
    if (nwg == 0) return CG_OK;
    ProfScope ps(c, s, kid, bytes, (double)nwg);
    // N = 8192: a launch with no more rows than compute units finishes a row sooner on 1024 threads
    const int e = (c->logn == 13 && nwg <= (size_t)c->n_cu) ? c->elems : c->elems_fwd;
    const int threads = c->N / e;
#define CG_FWD(LG, EL)                                                                          \
    do {                                                                                        \
        const unsigned grid = ntt_grid<ntt_fwd_kernel<LG, EL, LD, ST>>(c, nwg, threads);        \
        if (c->dry) return CG_OK;                                                               \
        return launch_kernel(ntt_fwd_kernel<LG, EL, LD, ST>, dim3(grid), dim3(threads), s, ld, st, \
                             (const double *)c->tw, (const DevConst *)c->dc, (int)nwg);         \
    } while (0)
    switch (c->logn * 100 + e) {
    case 1416: CG_FWD(14, 16);
    case 1208: CG_FWD(12, 8);
    case 1308: CG_FWD(13, 8);
    case 1316: CG_FWD(13, 16);
    default: return CG_EINVAL;
    }
#undef CG_FWD
}
template <class LD, class ST>
static int launch_inv(cg_ctx *c, hipStream_t s, size_t nwg, LD ld, ST st, int kid, double bytes)
{
    if (nwg == 0) return CG_OK;
    ProfScope ps(c, s, kid, bytes, (double)nwg);
    const int e = (c->logn == 13 && inv_wide<LD>::value) ? 16 : ntt_elems(c);
    const int threads = c->N / e;
#define CG_INV(LG, EL)                                                                          \
    do {                                                                                        \
        const unsigned grid = ntt_grid<ntt_inv_kernel<LG, EL, LD, ST>>(c, nwg, threads);        \
        if (c->dry) return CG_OK;                                                               \
        return launch_kernel(ntt_inv_kernel<LG, EL, LD, ST>, dim3(grid), dim3(threads), s, ld, st, \
                             (const double *)c->itw, (const DevConst *)c->dc, (int)nwg);        \
    } while (0)
    switch (c->logn * 100 + e) {
    case 1416: CG_INV(14, 16);
    case 1208: CG_INV(12, 8);
    case 1308: CG_INV(13, 8);
    case 1316: CG_INV(13, 16);
    default: return CG_EINVAL;
    }
#undef CG_INV
}
static unsigned pw_blocks(const cg_ctx *c, size_t rows) { return (unsigned)((rows * c->N + PW_THREADS - 1) / PW_THREADS); }
#define CG_TRY(expr) do { int rc_ = (expr); if (rc_ != CG_OK) return rc_; } while (0)

// ---------------------------------------------------------------------------
// internal operations (arguments already validated)
// ---------------------------------------------------------------------------
// one pointwise launch, bracketed by the timing scope
#define CG_LAUNCH_PW(kid, bytes, items, kernel, blocks, ...)                                                \
    do {                                                                                               \
        if (c->dry) break;                                                                             \
        int rc_pw_;                                                                                    \
        {                                                                                              \
            ProfScope ps_(c, s, kid, bytes, items);                                                    \
            rc_pw_ = launch_kernel(kernel, dim3(blocks), dim3(PW_THREADS), s, __VA_ARGS__);            \
        }                                                                                              \
        CG_TRY(rc_pw_);                                                                                \
    } while (0)

// mod-down of a summed series of rotations, one output row per workgroup
static int launch_moddown_sum(cg_ctx *c, hipStream_t s, double bytes, size_t batch, const ModdownArgs &A,
                              const ModdownHoist &H)
{
    if (c->dry) return CG_OK;
    ProfScope ps(c, s, KID_MODDOWN_SUM, bytes, (double)batch);
    const dim3 block(1024);
    const size_t rows = batch * 2 * c->k;
    const DevConst *dc = c->dc;
    switch (c->logn) {
    case 12: return launch_kernel(moddown_sum_kernel<12>, dim3((unsigned)(rows * moddown_sum_split<12>())), block, s, A, H, dc);
    case 13: return launch_kernel(moddown_sum_kernel<13>, dim3((unsigned)(rows * moddown_sum_split<13>())), block, s, A, H, dc);
    case 14: return launch_kernel(moddown_sum_kernel<14>, dim3((unsigned)(rows * moddown_sum_split<14>())), block, s, A, H, dc);
    default: return CG_EINVAL;
    }
}

// Every polynomial named by src -> its transform over the k ciphertext primes and the l auxiliary
// primes (centred lift), rows dst[poly][k+l][N], lazy.
static int transform_ext(cg_ctx *c, hipStream_t s, const MulSrc &src, size_t polys, double *dst)
{
    const double LB = (double)limb_bytes(c);
    const double in_rows = (double)polys * c->k;
    const StF64 st{dst, c->logn};
    CG_TRY(launch_fwd(c, s, polys * c->k, LdMulQ{src}, st, KID_FWD_MULQ, LB * 2.0 * in_rows));
    const double aux_bytes = LB * (in_rows + (double)polys * c->l);
    switch (c->k) {
    case 1: return launch_fwd(c, s, polys * c->l, LdMulAux<1>{src}, st, KID_FWD_MULB, aux_bytes);
    case 2: return launch_fwd(c, s, polys * c->l, LdMulAux<2>{src}, st, KID_FWD_MULB, aux_bytes);
    case 3: return launch_fwd(c, s, polys * c->l, LdMulAux<3>{src}, st, KID_FWD_MULB, aux_bytes);
    case 4: return launch_fwd(c, s, polys * c->l, LdMulAux<4>{src}, st, KID_FWD_MULB, aux_bytes);
    case 5: return launch_fwd(c, s, polys * c->l, LdMulAux<5>{src}, st, KID_FWD_MULB, aux_bytes);
    default: return launch_fwd(c, s, polys * c->l, LdMulAux<6>{src}, st, KID_FWD_MULB, aux_bytes);
    }
}

// Algorithmic bytes (distinct inputs read once + outputs written once) are attached to every
// launch for the roofline report; LB = bytes of one residue row.
// b ciphertext of unit u sits at index (u / b_group) * b_stride + u % b_group (b_group = 0: dense)
static int do_mul(cg_ctx *c, hipStream_t s, const uint64_t *a2, const uint64_t *b2, uint64_t *out3,
                  uint32_t batch, uint32_t a_group, void *ws, int accumulate, uint32_t b_group = 0,
                  uint32_t b_stride = 0, const double *b_ext = nullptr, uint32_t sum_group = 0)
{
    // b_ext: the b operands are already in transformed extended-basis form (cg_cache_extend);
    // only the a operands are transformed here
    // sum_group: the tensor products of every sum_group consecutive units are summed before the
    // inverse transform and the scaling; out3 then holds batch / sum_group results
    if (!b_group) { b_group = batch; b_stride = batch; }
    const uint32_t n_a = (batch + a_group - 1) / a_group;
    const size_t polys = 2 * ((size_t)n_a + (b_ext ? 0 : batch));
    Bump w = bump(c, ws);
    double *ntt = w.take<double>(polys * c->KL);
    double *tens = w.take<double>((size_t)3 * c->KL * batch);
    const double LB = (double)limb_bytes(c), B = batch;
    const MulSrc src{a2, b2, (int)n_a, (int)b_group, (int)b_stride, c->logn, 0};
    CG_TRY(transform_ext(c, s, src, polys, ntt));
    // tensor product fused into the inverse transform's load
    const LdInvTensor ld{ntt, b_ext, (int)a_group, (int)n_a, (int)b_group, (int)b_stride, c->logn};
    const uint32_t n_out = sum_group ? batch / sum_group : batch;
    const size_t rows = (size_t)n_out * 3 * c->KL;
    const double tbytes = LB * c->KL * (2.0 * ((double)n_a + B) + 3.0 * n_out);
    if (sum_group) CG_TRY(launch_inv(c, s, rows, LdInvTensorSum{ld, (int)sum_group}, StInvF64{tens, c->logn},
                                     KID_INV_TENSORSUM, tbytes));
    else CG_TRY(launch_inv(c, s, rows, ld, StInvF64{tens, c->logn}, KID_INV_TENSOR, tbytes));
    const double sbytes = LB * (3.0 * c->KL + 3.0 * c->k * (accumulate ? 2 : 1)) * n_out;
    const unsigned sblocks = pw_blocks(c, (size_t)n_out * 3);
#define CG_SCALE(K) CG_LAUNCH_PW(KID_SCALE, sbytes, (double)n_out, scale_kernel<K>, sblocks, tens, out3, (int)n_out * 3, accumulate, c->dc)
    switch (c->k) {
    case 1: CG_SCALE(1); break;
    case 2: CG_SCALE(2); break;
    case 3: CG_SCALE(3); break;
    case 4: CG_SCALE(4); break;
    case 5: CG_SCALE(5); break;
    default: CG_SCALE(6); break;
    }
#undef CG_SCALE
    return CG_OK;
}

// Mod-up of one ring element per unit (src + b*src_stride, Galois map first when galois != 0): the
// dnum digits extended to the k+nsp primes and transformed, rows dig[b][dnum][k+nsp][N]
static int launch_modup(cg_ctx *c, hipStream_t s, const uint64_t *src, size_t src_stride, uint32_t galois,
                        uint32_t batch, double *dig)
{
    const size_t nrows = (size_t)batch * c->dnum * c->L;
    const double mbytes = (double)limb_bytes(c) * (c->k + (double)c->dnum * c->L) * batch;
    const StF64 st{dig, c->logn};
#define CG_MODUP(G, A) return launch_fwd(c, s, nrows, LdModup<G, A>{src, src_stride, galois, c->logn}, st, KID_FWD_MODUP, mbytes)
    switch (c->alpha * 2 + (galois ? 1 : 0)) {
    case 2: CG_MODUP(false, 1);
    case 3: CG_MODUP(true, 1);
    case 4: CG_MODUP(false, 2);
    case 5: CG_MODUP(true, 2);
    case 6: CG_MODUP(false, 3);
    default: CG_MODUP(true, 3);
    }
#undef CG_MODUP
}

// key switch of one ring element per unit (src + b*src_stride), then the final additions
static int do_keyswitch(cg_ctx *c, hipStream_t s, const uint64_t *src, size_t src_stride, uint32_t galois,
                        const double *key, uint64_t *out2, size_t out_stride, const uint64_t *add, size_t add_stride,
                        uint32_t galois_inv, int accumulate, uint32_t batch, void *ws,
                        const uint64_t *acc_add = nullptr, size_t acc_stride = 0)
{
    if (!acc_add) { acc_add = add; acc_stride = add_stride; }
    Bump w = bump(c, ws);
    double *dig = w.take<double>((size_t)c->dnum * c->L * batch);
    double *acc = w.take<double>((size_t)2 * c->L * batch);
    const double LB = (double)limb_bytes(c), B = batch;
    const double dig_rows = (double)c->dnum * c->L;
    int rc;
    CG_TRY(launch_modup(c, s, src, src_stride, galois, batch, dig));
    // inner product with the key fused into the inverse transform's load
    const size_t irows = (size_t)batch * 2 * c->L;
    const double ibytes = LB * ((dig_rows + 2.0 * c->L) * B + 2.0 * dig_rows);
    const StInvF64 ist{acc, c->logn};
#define CG_KSI(D) launch_inv(c, s, irows, LdInvKsInner<D>{dig, key, c->logn}, ist, KID_INV_KSINNER, ibytes)
    switch (c->dnum) {
    case 1: rc = CG_KSI(1); break;
    case 2: rc = CG_KSI(2); break;
    case 3: rc = CG_KSI(3); break;
    case 4: rc = CG_KSI(4); break;
    case 5: rc = CG_KSI(5); break;
    default: rc = CG_KSI(6); break;
    }
#undef CG_KSI
    CG_TRY(rc);
    ModdownArgs A{acc, out2, out_stride, add, add_stride, galois_inv, accumulate, (int)batch, acc_add, acc_stride};
    const double add_rows = !add ? 0.0 : (galois_inv ? c->k + (accumulate ? 2.0 * c->k : 0.0) : 2.0 * c->k);
    CG_LAUNCH_PW(KID_MODDOWN, LB * (2.0 * c->L + add_rows + 2.0 * c->k) * B, B, moddown_kernel<false>,
                 pw_blocks(c, (size_t)batch * 2) / 2, A, ModdownHoist{}, c->dc);
    return CG_OK;
}

static int do_relin(cg_ctx *c, hipStream_t s, const uint64_t *in3, const void *rlk, uint64_t *out2, uint32_t batch,
                    void *ws)
{
    const size_t ct3 = (size_t)3 * c->k * c->N;
    return do_keyswitch(c, s, in3 + (size_t)2 * c->k * c->N, ct3, 0, static_cast<const double *>(rlk), out2,
                        (size_t)2 * c->k * c->N, in3, ct3, 0, 0, batch, ws);
}

static uint32_t inv_mod_pow2(uint32_t g, uint32_t two_n)
{
    uint32_t x = g;   // Newton iteration: correct to 3 bits, doubles each step
    for (int i = 0; i < 5; i++) x *= 2 - g * x;
    return x & (two_n - 1);
}

// in_stride / out_stride: uint64 between consecutive units (0 = densely packed ciphertexts)
// out2 = rotate(in2, g) (accumulate = 0), in2 + rotate(in2, g) (accumulate = 1, acc_add null) or
// acc_add + rotate(in2, g) (accumulate = 1, acc_add given; out2 may be acc_add itself)
static int do_rotate(cg_ctx *c, hipStream_t s, const uint64_t *in2, uint32_t g, const void *gk, uint64_t *out2,
                     uint32_t batch, int accumulate, void *ws, size_t in_stride = 0, size_t out_stride = 0,
                     const uint64_t *acc_add = nullptr, size_t acc_stride = 0)
{
    const size_t ct2 = (size_t)2 * c->k * c->N;
    if (!in_stride) in_stride = ct2;
    if (!out_stride) out_stride = ct2;
    return do_keyswitch(c, s, in2 + (size_t)c->k * c->N, in_stride, g, static_cast<const double *>(gk), out2,
                        out_stride, in2, in_stride, inv_mod_pow2(g, 2u * c->N), accumulate, batch, ws, acc_add,
                        acc_stride);
}

// A series of rotations of each of `batch` ciphertexts (in2 + b*in_stride): out2 + (b*out_per_b + i)
// ciphertexts receives rotation i (Galois element gs[i], prepared key keys[i]) in the hoisted form:
// one lift, extension and transform of the digits of c1, then per rotation a permuted inner
// product, inverse transforms and the mod-down with sigma_g(c0).  More than MAXROT rotations go in
// several rounds over the same digits.  ws: dnum (k+nsp) rows per ciphertext + 2 (k+nsp) rows per
// rotation of a round.
static int do_rotate_hoisted(cg_ctx *c, hipStream_t s, const uint64_t *in2, size_t in_stride, uint32_t n_rot,
                             const uint32_t *gs, const void *const *keys, uint64_t *out2, uint32_t out_per_b,
                             uint32_t batch, void *ws)
{
    const size_t ct2 = (size_t)2 * c->k * c->N;
    const double LB = (double)limb_bytes(c), B = batch;
    const double dig_rows = (double)c->dnum * c->L;
    const uint32_t round_max = n_rot < (uint32_t)MAXROT ? n_rot : (uint32_t)MAXROT;
    Bump w = bump(c, ws);
    double *dig = w.take<double>((size_t)c->dnum * c->L * batch);
    double *acc = w.take<double>((size_t)2 * c->L * batch * round_max);
    int rc;
    CG_TRY(launch_modup(c, s, in2 + (size_t)c->k * c->N, in_stride, 0, batch, dig));
    for (uint32_t i0 = 0; i0 < n_rot; i0 += MAXROT) {
        const uint32_t nr = n_rot - i0 < (uint32_t)MAXROT ? n_rot - i0 : (uint32_t)MAXROT;
        HoistTab T{};
        ModdownHoist H{};
        for (uint32_t i = 0; i < nr; i++) {
            T.g[i] = gs[i0 + i];
            T.key[i] = static_cast<const double *>(keys[i0 + i]);
            H.ginv[i] = inv_mod_pow2(gs[i0 + i], 2u * c->N);
        }
        H.rot_batch = (int)batch;
        H.out_per_b = (int)out_per_b;
        const size_t units = (size_t)batch * nr, irows = units * 2 * c->L;
        const double ibytes = LB * (dig_rows * B + 2.0 * c->L * units + 2.0 * dig_rows * nr);
        const StInvF64 ist{acc, c->logn};
#define CG_KSH(D) rc = launch_inv(c, s, irows, LdInvKsInnerHoisted<D>{dig, T, (int)batch, c->logn}, ist, KID_INV_KSINNER, ibytes)
        switch (c->dnum) {
        case 1: CG_KSH(1); break;
        case 2: CG_KSH(2); break;
        case 3: CG_KSH(3); break;
        case 4: CG_KSH(4); break;
        case 5: CG_KSH(5); break;
        default: CG_KSH(6); break;
        }
#undef CG_KSH
        CG_TRY(rc);
        // galois != 0 marks the rotation form; the element itself comes from the table
        ModdownArgs A{acc, out2 + (size_t)i0 * ct2, ct2, in2, in_stride, 1u, 0, (int)units, in2, in_stride};
        CG_LAUNCH_PW(KID_MODDOWN, LB * ((2.0 * c->L + 2.0 * c->k) * units + c->k * B), (double)units,
                     moddown_kernel<true>, pw_blocks(c, units * 2) / 2, A, H, c->dc);
    }
    return CG_OK;
}

// out2[b] = in2[b] + sum_i rotation i of in2[b] (Galois elements gs, prepared keys), the rotations
// hoisted and their key-switch accumulators summed before the one division by P.  in_stride /
// out_stride as in do_rotate.  ws: (dnum + 2)(k+nsp) rows per ciphertext.
static int do_rotate_sum(cg_ctx *c, hipStream_t s, const uint64_t *in2, size_t in_stride, uint32_t n_rot,
                         const uint32_t *gs, const void *const *keys, uint64_t *out2, size_t out_stride,
                         uint32_t batch, void *ws)
{
    const size_t ct2 = (size_t)2 * c->k * c->N;
    if (!in_stride) in_stride = ct2;
    if (!out_stride) out_stride = ct2;
    const double LB = (double)limb_bytes(c), B = batch;
    const double dig_rows = (double)c->dnum * c->L;
    Bump w = bump(c, ws);
    double *dig = w.take<double>((size_t)c->dnum * c->L * batch);
    double *acc = w.take<double>((size_t)2 * c->L * batch);
    int rc;
    CG_TRY(launch_modup(c, s, in2 + (size_t)c->k * c->N, in_stride, 0, batch, dig));
    HoistTab T{};
    ModdownHoist H{};
    for (uint32_t i = 0; i < n_rot; i++) {
        T.g[i] = gs[i];
        T.key[i] = static_cast<const double *>(keys[i]);
        H.ginv[i] = inv_mod_pow2(gs[i], 2u * c->N);
    }
    H.n_sum = (int)n_rot;
    const size_t irows = (size_t)batch * 2 * c->L;
    const double ibytes = LB * ((dig_rows + 2.0 * c->L) * B + 2.0 * dig_rows * n_rot);
    const StInvF64 ist{acc, c->logn};
#define CG_KSS(D) rc = launch_inv(c, s, irows, LdInvKsInnerSum<D>{dig, T, (int)n_rot, c->logn}, ist, KID_INV_KSSUM, ibytes)
    switch (c->dnum) {
    case 1: CG_KSS(1); break;
    case 2: CG_KSS(2); break;
    case 3: CG_KSS(3); break;
    case 4: CG_KSS(4); break;
    case 5: CG_KSS(5); break;
    default: CG_KSS(6); break;
    }
#undef CG_KSS
    CG_TRY(rc);
    ModdownArgs A{acc, out2, out_stride, in2, in_stride, 1u, 1, (int)batch, in2, in_stride};
    // reads: the accumulators and the ciphertext (the permuted reads of c0 come from LDS)
    return launch_moddown_sum(c, s, LB * (2.0 * c->L + 4.0 * c->k) * B, batch, A, H);
}

static int do_add(cg_ctx *c, hipStream_t s, const uint64_t *a, const uint64_t *b, uint64_t *out, size_t rows)
{
    CG_LAUNCH_PW(KID_ADD, (double)limb_bytes(c) * 3.0 * rows, (double)rows, add_kernel, pw_blocks(c, rows), a, b, out, (int)rows,
                 c->dc);
    return CG_OK;
}

static bool ptrs_ok(std::initializer_list<const void *> ps)
{
    for (const void *p : ps) if (!p || !aligned16(p)) return false;
    return true;
}
// two device ranges share at least one byte
static bool overlap(const void *a, size_t a_bytes, const void *b, size_t b_bytes)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + b_bytes && y < x + a_bytes;
}
static bool overlap(const void *a, const void *b, size_t bytes) { return overlap(a, bytes, b, bytes); }
static bool batch_ok(uint32_t batch) { return batch >= 1 && batch <= (1u << 16); }
static bool galois_ok(const cg_ctx *c, uint32_t g) { return (g & 1) && g > 0 && g < 2u * c->N; }

// ---------------------------------------------------------------------------
// public entry points
// ---------------------------------------------------------------------------
static int public_transform(cg_ctx *c, void *stream, const uint64_t *in, uint64_t *out, const uint32_t *idx,
                            uint32_t n_limbs, bool inverse)
{
    CG_REQUIRE(c && idx && ptrs_ok({in, out}) && n_limbs >= 1 && n_limbs <= c->tab_cap);
    for (uint32_t i = 0; i < n_limbs; i++) CG_REQUIRE(idx[i] < (uint32_t)c->L);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The usual pattern -- row i modulo prime i % period, as in stacked ring elements -- needs no
    // table.  Any other assignment is staged through a context-owned device buffer; that copy
    // is ordered on the caller's stream before the kernel.
    uint32_t period = 0;
    for (uint32_t i = 0; i < n_limbs; i++) if (idx[i] >= period) period = idx[i] + 1;
    bool periodic = true;
    for (uint32_t i = 0; i < n_limbs && periodic; i++) periodic = idx[i] == i % period;
    const uint32_t *tab = nullptr;
    if (!periodic) {
        // the table is copied from the caller's (pageable) host array when the call is made, not when
        // a captured graph replays: refuse that form on a capturing stream
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        CG_HIP(hipStreamIsCapturing(s, &cap));
        CG_REQUIRE(cap == hipStreamCaptureStatusNone);
        CG_HIP(hipMemcpyAsync(c->tab, idx, n_limbs * sizeof(uint32_t), hipMemcpyHostToDevice, s));
        tab = c->tab;
    }
    if (!inverse)
        return launch_fwd(c, s, n_limbs, LdRowsU64{in, tab, (int)period, c->logn}, StU64{out, c->logn}, KID_FWD_ROWS,
                          2.0 * limb_bytes(c) * n_limbs);
    return launch_inv(c, s, n_limbs, LdInvU64{in, tab, (int)period, c->logn}, StInvU64{out, c->logn}, KID_INV_U64,
                      2.0 * limb_bytes(c) * n_limbs);
}
extern "C" int cg_ntt_forward(cg_ctx *c, void *stream, const uint64_t *in, uint64_t *out, const uint32_t *idx,
                              uint32_t n_limbs)
{
    return public_transform(c, stream, in, out, idx, n_limbs, false);
}
extern "C" int cg_ntt_inverse(cg_ctx *c, void *stream, const uint64_t *in, uint64_t *out, const uint32_t *idx,
                              uint32_t n_limbs)
{
    return public_transform(c, stream, in, out, idx, n_limbs, true);
}

extern "C" int cg_ksk_prepare(cg_ctx *c, void *stream, const uint64_t *raw, void *ksk)
{
    CG_REQUIRE(c && ptrs_ok({raw, ksk}));
    return launch_fwd(c, static_cast<hipStream_t>(stream), (size_t)c->dnum * 2 * c->L,
                      LdRowsU64{raw, nullptr, c->L, c->logn}, StF64Red{static_cast<double *>(ksk), c->logn},
                      KID_FWD_ROWS, 4.0 * limb_bytes(c) * c->dnum * c->L);
}

extern "C" int cg_plain_prepare(cg_ctx *c, void *stream, const uint64_t *pt, void *plain, uint32_t batch)
{
    CG_REQUIRE(c && ptrs_ok({pt, plain}) && batch_ok(batch));
    return launch_fwd(c, static_cast<hipStream_t>(stream), (size_t)batch * c->k, LdPlain{pt, c->logn},
                      StF64Red{static_cast<double *>(plain), c->logn}, KID_FWD_PLAIN,
                      (double)limb_bytes(c) * batch * (1.0 + c->k));
}

extern "C" int cg_mul(cg_ctx *c, void *stream, const uint64_t *a2, const uint64_t *b2, uint64_t *out3,
                      uint32_t batch, uint32_t a_group, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({a2, b2, out3, ws}) && batch_ok(batch) && a_group >= 1);
    return do_mul(c, static_cast<hipStream_t>(stream), a2, b2, out3, batch, a_group, ws, 0);
}

extern "C" int cg_mul_sum(cg_ctx *c, void *stream, const uint64_t *a2, const uint64_t *b2, uint64_t *out3,
                          uint32_t n_groups, uint32_t group_len, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({a2, b2, out3, ws}) && n_groups >= 1 && group_len >= 1);
    CG_REQUIRE((uint64_t)n_groups * group_len <= (1u << 16));
    return do_mul(c, static_cast<hipStream_t>(stream), a2, b2, out3, n_groups * group_len, 1, ws, 0, 0, 0, nullptr,
                  group_len);
}

extern "C" int cg_relin(cg_ctx *c, void *stream, const uint64_t *in3, const void *rlk, uint64_t *out2,
                        uint32_t batch, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({in3, rlk, out2, ws}) && batch_ok(batch));
    return do_relin(c, static_cast<hipStream_t>(stream), in3, rlk, out2, batch, ws);
}

extern "C" int cg_mul_relin(cg_ctx *c, void *stream, const uint64_t *a2, const uint64_t *b2, const void *rlk,
                            uint64_t *out2, uint32_t batch, uint32_t a_group, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({a2, b2, rlk, out2, ws}) && batch_ok(batch) && a_group >= 1);
    hipStream_t s = static_cast<hipStream_t>(stream);
    Bump w = bump(c, ws);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    CG_TRY(do_mul(c, s, a2, b2, d3, batch, a_group, w.p, 0));
    return do_relin(c, s, d3, rlk, out2, batch, w.p);
}

extern "C" size_t cg_static_scratch_bytes(void) { return CG_STATIC_SCRATCH_BYTES; }

// cg_mul_relin on the library's own scratch array: no allocation, by this call or by anything it
// calls (launches and, with profiling on, event records only)
extern "C" int cg_mul_relin_static(cg_ctx *c, void *stream, const uint64_t *a2, const uint64_t *b2, const void *rlk,
                                   uint64_t *out2, uint32_t batch, uint32_t a_group)
{
    CG_REQUIRE(c && ptrs_ok({a2, b2, rlk, out2}) && batch_ok(batch) && a_group >= 1);
    if (cg_workspace_bytes(c, batch) > (size_t)CG_STATIC_SCRATCH_BYTES) return CG_ESCRATCH;
    int dev = -1;
    CG_HIP(hipGetDevice(&dev));
    CG_REQUIRE(dev == c->device && c->static_ws);   // the array's address differs from GPU to GPU
    return cg_mul_relin(c, stream, a2, b2, rlk, out2, batch, a_group, c->static_ws);
}

extern "C" int cg_rotate(cg_ctx *c, void *stream, const uint64_t *in2, uint32_t g, const void *gk, uint64_t *out2,
                         uint32_t batch, int accumulate, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({in2, gk, out2, ws}) && batch_ok(batch) && galois_ok(c, g));
    CG_REQUIRE(!overlap(in2, out2, (size_t)batch * 2 * c->k * limb_bytes(c)));
    return do_rotate(c, static_cast<hipStream_t>(stream), in2, g, gk, out2, batch, accumulate, ws);
}

static bool rot_series_ok(const cg_ctx *c, uint32_t n_rot, const uint32_t *gs, const void *const *keys)
{
    if (!gs || !keys || n_rot < 1 || n_rot > 4096) return false;
    for (uint32_t i = 0; i < n_rot; i++)
        if (!galois_ok(c, gs[i]) || !keys[i] || !aligned16(keys[i])) return false;
    return true;
}

extern "C" int cg_rotate_hoisted(cg_ctx *c, void *stream, const uint64_t *in2, uint32_t n_rot, const uint32_t *gs,
                                 const void *const *gks, uint64_t *out2, uint32_t batch, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({in2, out2, ws}) && batch_ok(batch) && rot_series_ok(c, n_rot, gs, gks));
    CG_REQUIRE((uint64_t)batch * n_rot <= (1u << 16));
    const size_t ct2b = (size_t)2 * c->k * limb_bytes(c);
    CG_REQUIRE(!overlap(in2, ct2b * batch, out2, ct2b * batch * n_rot));
    return do_rotate_hoisted(c, static_cast<hipStream_t>(stream), in2, (size_t)2 * c->k * c->N, n_rot, gs, gks, out2,
                             n_rot, batch, ws);
}

extern "C" int cg_rotate_sum_hoisted(cg_ctx *c, void *stream, const uint64_t *in2, uint32_t n_rot, const uint32_t *gs,
                                     const void *const *gks, uint64_t *out2, uint32_t batch, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({in2, out2, ws}) && batch_ok(batch) && rot_series_ok(c, n_rot, gs, gks));
    CG_REQUIRE(n_rot <= (uint32_t)MAXROT);
    const size_t ct2b = (size_t)2 * c->k * limb_bytes(c);
    CG_REQUIRE(!overlap(in2, ct2b * batch, out2, ct2b * batch));
    return do_rotate_sum(c, static_cast<hipStream_t>(stream), in2, 0, n_rot, gs, gks, out2, 0, batch, ws);
}

extern "C" int cg_add(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *b, uint64_t *out, uint32_t ncomp,
                      uint32_t batch)
{
    CG_REQUIRE(c && ptrs_ok({a, b, out}) && batch_ok(batch) && (ncomp == 2 || ncomp == 3));
    return do_add(c, static_cast<hipStream_t>(stream), a, b, out, (size_t)batch * ncomp * c->k);
}

extern "C" int cg_add_plain(cg_ctx *c, void *stream, const uint64_t *in2, const uint64_t *pt, uint32_t n_plain,
                            int negative, uint64_t *out2, uint32_t batch)
{
    CG_REQUIRE(c && ptrs_ok({in2, pt, out2}) && batch_ok(batch) && n_plain >= 1 && n_plain <= batch);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t rows = (size_t)batch * 2 * c->k;
    CG_LAUNCH_PW(KID_ADD, (double)limb_bytes(c) * (2.0 * rows + n_plain), (double)rows, add_plain_kernel, pw_blocks(c, rows), in2, pt,
                 out2, (int)batch, (int)n_plain, negative ? 1 : 0, c->dc);
    return CG_OK;
}

extern "C" int cg_mul_plain(cg_ctx *c, void *stream, const uint64_t *in2, const void *plain, uint32_t plain_stride,
                            uint64_t *out2, uint32_t batch, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({in2, plain, out2, ws}) && batch_ok(batch));
    hipStream_t s = static_cast<hipStream_t>(stream);
    double *f = static_cast<double *>(ws);
    const size_t rows = (size_t)batch * 2 * c->k;
    const double LB = (double)limb_bytes(c);
    CG_TRY(launch_fwd(c, s, rows, LdRowsU64{in2, nullptr, c->k, c->logn}, StF64{f, c->logn}, KID_FWD_ROWS,
                      LB * 2.0 * rows));
    return launch_inv(c, s, rows,
                      LdInvMulPlain{f, static_cast<const double *>(plain), 1, 1 << 30, (int)plain_stride, 0, c->logn},
                      StInvU64{out2, c->logn}, KID_INV_MULPLAIN,
                      LB * (2.0 * rows + c->k * (plain_stride ? (double)batch : 1.0)));
}

extern "C" int cg_kv_append(cg_ctx *c, void *stream, uint64_t *cache, uint32_t cache_stride_cts, uint32_t n_caches,
                            uint32_t tau, const uint64_t *rows_dev, const void *masks, uint32_t d2, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({cache, rows_dev, masks, ws}) && batch_ok(n_caches));
    CG_REQUIRE(d2 >= 1 && (d2 & (d2 - 1)) == 0 && d2 <= (uint32_t)c->N / 2);
    const uint32_t B = (uint32_t)c->N / d2, ct_idx = tau / B, blk = tau % B;
    CG_REQUIRE(ct_idx < cache_stride_cts);
    hipStream_t s = static_cast<hipStream_t>(stream);
    double *f = static_cast<double *>(ws);
    const size_t rows = (size_t)n_caches * 2 * c->k;
    const size_t ct2 = (size_t)2 * c->k * c->N;
    const double LB = (double)limb_bytes(c);
    CG_TRY(launch_fwd(c, s, rows, LdRowsU64{rows_dev, nullptr, c->k, c->logn}, StF64{f, c->logn}, KID_FWD_ROWS,
                      LB * 2.0 * rows));
    return launch_inv(c, s, rows, LdInvMulPlain{f, static_cast<const double *>(masks), 1, 1 << 30, 0, (int)blk, c->logn},
                      StInvAppend{cache + (size_t)ct_idx * ct2, (size_t)cache_stride_cts * ct2, blk == 0 ? 1 : 0,
                                  c->logn},
                      KID_INV_MULPLAIN, LB * ((blk == 0 ? 2.0 : 3.0) * rows + c->k));
}

static bool pow2_d(const cg_ctx *c, uint32_t d2) { return d2 >= 2 && (d2 & (d2 - 1)) == 0 && d2 <= (uint32_t)c->N / 4; }
static uint32_t pow3_mod(uint32_t e, uint32_t two_n)
{
    uint64_t r = 1, b = 3;
    for (; e; e >>= 1, b = b * b % two_n)
        if (e & 1) r = r * b % two_n;
    return (uint32_t)r;
}

// x <- x + rotate(x, g) for each g of the list, ping-ponging between two buffers;
// the last result lands in `out`.  x0 holds the start value.
static int rotate_add_chain(cg_ctx *c, hipStream_t s, uint64_t *x0, uint64_t *x1, uint64_t *out,
                            const uint32_t *gs, const void *const *keys, int n, uint32_t batch, void *ws)
{
    uint64_t *cur = x0, *nxt = x1;
    for (int i = 0; i < n; i++) {
        uint64_t *dst = (i == n - 1) ? out : nxt;
        CG_TRY(do_rotate(c, s, cur, gs[i], keys[i], dst, batch, 1, ws));
        nxt = cur;
        cur = dst;
    }
    return CG_OK;
}

// A folding sum over the subset products of the generators gens[0 .. n_bits) taken in rounds:
// ceil(n_bits / w) rounds of as even a number of bits as possible, the longer ones first; a round
// over bits [b0, b0 + c) adds to its input its rotations by the 2^c - 1 products of non-empty
// subsets of gens[b0 .. b0 + c) (entry m - 1: the generators whose bit is set in m), hoisted, with
// one mod-down.  keys: the prepared keys of all rounds in that order.
struct FoldRounds {
    int n_rounds = 0, n_keys = 0;
    int first[16], count[16];
    std::vector<uint32_t> g;
};
static bool fold_rounds(const cg_ctx *c, const uint32_t *gens, int n_bits, uint32_t w, FoldRounds &R)
{
    if (w < 1 || w > 7 || n_bits < 0 || n_bits > 16) return false;   // 2^7 - 1 rotations fit one launch
    if (!n_bits) return true;
    const int rounds = (n_bits + (int)w - 1) / (int)w, lo = n_bits / rounds, extra = n_bits % rounds;
    int b0 = 0;
    for (int r = 0; r < rounds; r++) {
        const int cb = lo + (r < extra ? 1 : 0);
        R.first[r] = R.n_keys;
        R.count[r] = (1 << cb) - 1;
        for (uint32_t m = 1; m < (1u << cb); m++) {
            uint64_t e = 1;
            for (int i = 0; i < cb; i++)
                if ((m >> i) & 1) e = e * gens[b0 + i] % (2u * c->N);
            R.g.push_back((uint32_t)e);
        }
        R.n_keys += R.count[r];
        b0 += cb;
    }
    R.n_rounds = rounds;
    return true;
}
static bool fold_keys_ok(const FoldRounds &R, const void *const *keys)
{
    if (R.n_keys && !keys) return false;
    for (int i = 0; i < R.n_keys; i++)
        if (!keys[i] || !aligned16(keys[i])) return false;
    return true;
}
// x0 holds the start value; rounds ping-pong between x0 and x1, the last result lands in `out`
static int fold_chain(cg_ctx *c, hipStream_t s, uint64_t *x0, uint64_t *x1, uint64_t *out, const FoldRounds &R,
                      const void *const *keys, uint32_t batch, void *ws)
{
    uint64_t *cur = x0, *nxt = x1;
    for (int r = 0; r < R.n_rounds; r++) {
        uint64_t *dst = (r == R.n_rounds - 1) ? out : nxt;
        CG_TRY(do_rotate_sum(c, s, cur, 0, (uint32_t)R.count[r], R.g.data() + R.first[r], keys + R.first[r], dst, 0,
                             batch, ws));
        nxt = cur;
        cur = dst;
    }
    return CG_OK;
}

// generators of the two folding sums: the slots of a block (scores), the blocks and the two rows (context)
static int fold_generators(const cg_ctx *c, uint32_t d2, uint32_t *gs)
{
    int n = 0;
    for (uint32_t sh = 1; sh < d2; sh <<= 1) gs[n++] = pow3_mod(sh, 2u * c->N);
    return n;
}
static int block_generators(const cg_ctx *c, uint32_t d2, uint32_t *gs)
{
    int n = 0;
    for (uint32_t sh = d2; sh <= (uint32_t)c->N / 4; sh <<= 1) gs[n++] = pow3_mod(sh, 2u * c->N);
    gs[n++] = 2u * c->N - 1;
    return n;
}

extern "C" int cg_round_galois(const cg_ctx *c, int which, uint32_t d2, uint32_t round_bits, uint32_t *elts_host,
                               uint32_t cap, uint32_t *n_out)
{
    CG_REQUIRE(c && n_out && (which == 0 || which == 1) && pow2_d(c, d2) && (elts_host || !cap));
    uint32_t gs[20];
    const int nb = which ? block_generators(c, d2, gs) : fold_generators(c, d2, gs);
    FoldRounds R;
    CG_REQUIRE(fold_rounds(c, gs, nb, round_bits, R));
    for (uint32_t i = 0; i < cap && i < (uint32_t)R.n_keys; i++) elts_host[i] = R.g[i];
    *n_out = (uint32_t)R.n_keys;
    return CG_OK;
}

// kext != null: the cache in transformed form (kc is then not read)
// w != 0: the folding sum in rounds of w bits (fold_rounds), gk_fold holding the rounds' keys
static int scores_impl(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kc, const double *kext,
                       uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                       const void *const *gk_fold, uint64_t *out, void *ws, uint32_t fold_w = 0)
{
    CG_REQUIRE(c && ptrs_ok({q, kext ? (const void *)kext : (const void *)kc, rlk, out, ws}) && gk_fold &&
               heads >= 1 && n_cts >= 1 && pow2_d(c, d2));
    CG_REQUIRE(cache_stride_cts >= n_cts);
    const uint32_t batch = heads * n_cts;
    CG_REQUIRE(batch_ok(batch));
    uint32_t gs[20];
    const int nrot = fold_generators(c, d2, gs);
    FoldRounds R;
    if (fold_w) {
        CG_REQUIRE(fold_rounds(c, gs, nrot, fold_w, R) && fold_keys_ok(R, gk_fold));
    } else {
        for (int i = 0; i < nrot; i++) CG_REQUIRE(gk_fold[i] && aligned16(gk_fold[i]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Bump w = bump(c, ws);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    uint64_t *xa = w.take<uint64_t>((size_t)2 * c->k * batch), *xb = w.take<uint64_t>((size_t)2 * c->k * batch);
    CG_TRY(do_mul(c, s, q, kc, d3, batch, n_cts, w.p, 0, n_cts, cache_stride_cts, kext));
    CG_TRY(do_relin(c, s, d3, rlk, xa, batch, w.p));
    if (fold_w) return fold_chain(c, s, xa, xb, out, R, gk_fold, batch, w.p);
    return rotate_add_chain(c, s, xa, xb, out, gs, gk_fold, nrot, batch, w.p);
}
extern "C" int cg_decode_scores(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kc, uint32_t heads,
                                uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                                const void *const *gk_fold, uint64_t *out, void *ws)
{
    return scores_impl(c, stream, q, kc, nullptr, heads, n_cts, cache_stride_cts, d2, rlk, gk_fold, out, ws);
}
extern "C" int cg_decode_scores_ext(cg_ctx *c, void *stream, const uint64_t *q, const void *kext, uint32_t heads,
                                    uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                                    const void *const *gk_fold, uint64_t *out, void *ws)
{
    CG_REQUIRE(kext);
    return scores_impl(c, stream, q, nullptr, static_cast<const double *>(kext), heads, n_cts, cache_stride_cts, d2,
                       rlk, gk_fold, out, ws);
}

static int context_impl(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *vc, const double *vext,
                        uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                        const void *const *gk_block, uint64_t *out, void *ws, uint32_t fold_w = 0,
                        bool sum_first = false)
{
    CG_REQUIRE(c && ptrs_ok({a, vext ? (const void *)vext : (const void *)vc, rlk, out, ws}) && gk_block &&
               heads >= 1 && n_cts >= 1 && pow2_d(c, d2));
    CG_REQUIRE(cache_stride_cts >= n_cts);
    const uint32_t batch = heads * n_cts;
    CG_REQUIRE(batch_ok(batch));
    uint32_t gs[20];
    const int nrot = block_generators(c, d2, gs);
    FoldRounds R;
    if (fold_w) {
        CG_REQUIRE(fold_rounds(c, gs, nrot, fold_w, R) && fold_keys_ok(R, gk_block));
    } else {
        for (int i = 0; i < nrot; i++) CG_REQUIRE(gk_block[i] && aligned16(gk_block[i]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Bump w = bump(c, ws);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    uint64_t *y = w.take<uint64_t>((size_t)3 * c->k * heads);
    uint64_t *xa = w.take<uint64_t>((size_t)2 * c->k * heads), *xb = w.take<uint64_t>((size_t)2 * c->k * heads);
    if (sum_first) {
        // y[h] = one scaling of the sum over c of the tensor products
        CG_TRY(do_mul(c, s, a, vc, y, batch, 1, w.p, 0, n_cts, cache_stride_cts, vext, n_cts));
    } else {
        CG_TRY(do_mul(c, s, a, vc, d3, batch, 1, w.p, 0, n_cts, cache_stride_cts, vext));
        // y[h] = sum_c d3[h][c]  (three components)
        const int rows = 3 * c->k;
        CG_LAUNCH_PW(KID_SUM_GROUPS, (double)limb_bytes(c) * rows * (batch + heads), (double)batch, sum_groups_kernel,
                     pw_blocks(c, (size_t)heads * rows), d3, y, (int)heads, (int)n_cts, rows, c->dc);
    }
    CG_TRY(do_relin(c, s, y, rlk, xa, heads, w.p));
    if (fold_w) return fold_chain(c, s, xa, xb, out, R, gk_block, heads, w.p);
    return rotate_add_chain(c, s, xa, xb, out, gs, gk_block, nrot, heads, w.p);
}
extern "C" int cg_decode_context(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *vc, uint32_t heads,
                                 uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                                 const void *const *gk_block, uint64_t *out, void *ws)
{
    return context_impl(c, stream, a, vc, nullptr, heads, n_cts, cache_stride_cts, d2, rlk, gk_block, out, ws);
}
extern "C" int cg_decode_context_ext(cg_ctx *c, void *stream, const uint64_t *a, const void *vext, uint32_t heads,
                                     uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, const void *rlk,
                                     const void *const *gk_block, uint64_t *out, void *ws)
{
    CG_REQUIRE(vext);
    return context_impl(c, stream, a, nullptr, static_cast<const double *>(vext), heads, n_cts, cache_stride_cts, d2,
                        rlk, gk_block, out, ws);
}

extern "C" int cg_decode_scores_hoisted(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kc, const void *kext,
                                        uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                                        uint32_t round_bits, const void *rlk, const void *const *gk_rounds,
                                        uint64_t *out, void *ws)
{
    CG_REQUIRE(round_bits >= 1);
    return scores_impl(c, stream, q, kext ? nullptr : kc, static_cast<const double *>(kext), heads, n_cts,
                       cache_stride_cts, d2, rlk, gk_rounds, out, ws, round_bits);
}
extern "C" int cg_decode_context_hoisted(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *vc, const void *vext,
                                         uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2,
                                         uint32_t round_bits, int sum_before_scaling, const void *rlk,
                                         const void *const *gk_rounds, uint64_t *out, void *ws)
{
    CG_REQUIRE(round_bits >= 1 && (sum_before_scaling == 0 || sum_before_scaling == 1));
    return context_impl(c, stream, a, vext ? nullptr : vc, static_cast<const double *>(vext), heads, n_cts,
                        cache_stride_cts, d2, rlk, gk_rounds, out, ws, round_bits, sum_before_scaling != 0);
}

extern "C" int cg_cache_extend(cg_ctx *c, void *stream, const uint64_t *cts, uint32_t n_groups, uint32_t group_len,
                               uint32_t group_stride_cts, void *ext)
{
    CG_REQUIRE(c && ptrs_ok({cts, ext}) && n_groups >= 1 && group_len >= 1 && group_stride_cts >= group_len);
    CG_REQUIRE((uint64_t)n_groups * group_len <= (1u << 16));
    const MulSrc src{nullptr, cts, 0, (int)group_len, (int)group_stride_cts, c->logn, 1};
    return transform_ext(c, static_cast<hipStream_t>(stream), src, (size_t)2 * n_groups * group_len,
                         static_cast<double *>(ext));
}

extern "C" size_t cg_decode_step_workspace_bytes(const cg_ctx *c, uint32_t heads, uint32_t n_cts)
{
    if (!c || !heads || !n_cts || (uint64_t)heads * n_cts > (1u << 16)) return 0;
    return 2 * cg_workspace_bytes(c, heads * n_cts) + cg_workspace_bytes(c, 2 * heads);
}

// ext != null: the cache's transformed copy is read by the products and brought up to date for
// the appended ciphertext of every cache
static int step_impl(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *a, uint64_t *cache, double *ext,
                     uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, uint32_t tau,
                     const uint64_t *rows, const void *masks, const void *rlk, const void *const *gk_fold,
                     const void *const *gk_block, uint64_t *scores, uint64_t *context, void *ws,
                     uint32_t fold_w = 0, uint32_t block_w = 0, bool sum_first = false)
{
    CG_REQUIRE(c && ptrs_ok({q, a, cache, rows, masks, rlk, scores, context, ws}) && gk_fold && gk_block);
    CG_REQUIRE(heads >= 1 && n_cts >= 1 && batch_ok(heads * n_cts) && pow2_d(c, d2) && cache_stride_cts >= n_cts);
    CG_REQUIRE(tau / ((uint32_t)c->N / d2) < cache_stride_cts);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t ct2 = (size_t)2 * c->k * c->N;
    uint64_t *vcache = cache + (size_t)heads * cache_stride_cts * ct2;
    char *ws_scores = static_cast<char *>(ws);
    char *ws_context = ws_scores + cg_workspace_bytes(c, heads * n_cts);
    char *ws_append = ws_context + cg_workspace_bytes(c, heads * n_cts);
    const size_t ext_ct = (size_t)2 * c->KL * c->N;          // doubles per transformed ciphertext
    const uint32_t app_idx = tau / ((uint32_t)c->N / d2);
    const double *kext = ext, *vext = ext ? ext + (size_t)heads * cache_stride_cts * ext_ct : nullptr;
    // append, then (with a transformed copy) re-transform the ciphertext every cache just received
    auto append = [&](hipStream_t st) -> int {
        CG_TRY(cg_kv_append(c, st, cache, cache_stride_cts, 2 * heads, tau, rows, masks, d2, ws_append));
        if (!ext) return CG_OK;
        return cg_cache_extend(c, st, cache + (size_t)app_idx * ct2, 2 * heads, 1, cache_stride_cts,
                               ext + (size_t)app_idx * ext_ct);
    };
    // The appended ciphertext is read by this step's products only when it lies inside the first
    // n_cts: then the append goes first on the caller's stream; otherwise it is a third branch.
    const bool append_first = tau / ((uint32_t)c->N / d2) < n_cts;
    if (append_first) CG_TRY(append(s));
    CG_HIP(hipEventRecord(c->ev_fork, s));
    CG_HIP(hipStreamWaitEvent(c->side[0], c->ev_fork, 0));
    if (!append_first) CG_HIP(hipStreamWaitEvent(c->side[1], c->ev_fork, 0));
    // Branches are always joined, also after a failed launch, so that the caller's stream never
    // runs ahead of work this call started.
    int rc = scores_impl(c, s, q, cache, kext, heads, n_cts, cache_stride_cts, d2, rlk, gk_fold, scores, ws_scores,
                         fold_w);
    const int rc1 = context_impl(c, c->side[0], a, vcache, vext, heads, n_cts, cache_stride_cts, d2, rlk, gk_block,
                                 context, ws_context, block_w, sum_first);
    if (rc == CG_OK) rc = rc1;
    if (!append_first) {
        const int rc2 = append(c->side[1]);
        if (rc == CG_OK) rc = rc2;
    }
    for (int i = 0; i < (append_first ? 1 : 2); i++) {
        CG_HIP(hipEventRecord(c->ev_join[i], c->side[i]));
        CG_HIP(hipStreamWaitEvent(s, c->ev_join[i], 0));
    }
    return rc;
}

extern "C" int cg_decode_step(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *a, uint64_t *cache,
                              uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts, uint32_t d2, uint32_t tau,
                              const uint64_t *rows, const void *masks, const void *rlk, const void *const *gk_fold,
                              const void *const *gk_block, uint64_t *scores, uint64_t *context, void *ws)
{
    return step_impl(c, stream, q, a, cache, nullptr, heads, n_cts, cache_stride_cts, d2, tau, rows, masks, rlk, gk_fold,
                     gk_block, scores, context, ws);
}
extern "C" int cg_decode_step_ext(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *a, uint64_t *cache,
                                  void *cache_ext, uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts,
                                  uint32_t d2, uint32_t tau, const uint64_t *rows, const void *masks, const void *rlk,
                                  const void *const *gk_fold, const void *const *gk_block, uint64_t *scores,
                                  uint64_t *context, void *ws)
{
    CG_REQUIRE(cache_ext && aligned16(cache_ext));
    return step_impl(c, stream, q, a, cache, static_cast<double *>(cache_ext), heads, n_cts, cache_stride_cts, d2, tau,
                     rows, masks, rlk, gk_fold, gk_block, scores, context, ws);
}

extern "C" int cg_decode_step_hoisted(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *a, uint64_t *cache,
                                      void *cache_ext, uint32_t heads, uint32_t n_cts, uint32_t cache_stride_cts,
                                      uint32_t d2, uint32_t tau, const uint64_t *rows, const void *masks,
                                      const void *rlk, uint32_t fold_round_bits, const void *const *gk_fold_rounds,
                                      uint32_t block_round_bits, int sum_before_scaling,
                                      const void *const *gk_block_rounds, uint64_t *scores, uint64_t *context, void *ws)
{
    CG_REQUIRE(fold_round_bits >= 1 && block_round_bits >= 1 && (!cache_ext || aligned16(cache_ext)));
    CG_REQUIRE(sum_before_scaling == 0 || sum_before_scaling == 1);
    return step_impl(c, stream, q, a, cache, static_cast<double *>(cache_ext), heads, n_cts, cache_stride_cts, d2, tau,
                     rows, masks, rlk, gk_fold_rounds, gk_block_rounds, scores, context, ws, fold_round_bits,
                     block_round_bits, sum_before_scaling != 0);
}

extern "C" int cg_decode_scores_outer(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kcols,
                                      uint32_t heads, uint32_t d2, const void *masks, const void *rlk,
                                      const void *const *gk_fold, uint64_t *out, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({q, kcols, masks, rlk, out, ws}) && gk_fold && heads >= 1 && pow2_d(c, d2));
    const uint32_t batch = heads * d2;
    CG_REQUIRE(batch_ok(batch));
    int nrot = 0;
    uint32_t gs[16];
    for (uint32_t sh = 1; sh < d2; sh <<= 1) {
        CG_REQUIRE(gk_fold[nrot] && aligned16(gk_fold[nrot]));
        gs[nrot++] = pow3_mod(sh, 2u * c->N);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const double LB = (double)limb_bytes(c);
    Bump w = bump(c, ws);
    uint64_t *xa = w.take<uint64_t>((size_t)2 * c->k * batch), *xb = w.take<uint64_t>((size_t)2 * c->k * batch);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    uint64_t *y = w.take<uint64_t>((size_t)3 * c->k * heads);
    // x[h][j] = q[h] * mask_j: one forward transform per query row, the mask product rides on the
    // inverse transform's load
    double *f = reinterpret_cast<double *>(d3);   // free until the products are formed
    const size_t qrows = (size_t)heads * 2 * c->k, xrows = (size_t)batch * 2 * c->k;
    CG_TRY(launch_fwd(c, s, qrows, LdRowsU64{q, nullptr, c->k, c->logn}, StF64{f, c->logn}, KID_FWD_ROWS,
                      LB * 2.0 * qrows));
    CG_TRY(launch_inv(c, s, xrows,
                      LdInvMulPlain{f, static_cast<const double *>(masks), (int)d2, (int)d2, 1, 0, c->logn},
                      StInvU64{xa, c->logn}, KID_INV_MULPLAIN, LB * (qrows + (double)d2 * c->k + xrows)));
    // broadcast q_j to every slot: log2(d2) rotate-and-add steps; the last one lands in xb or xa
    uint64_t *bc = (nrot & 1) ? xb : xa;
    if (nrot) CG_TRY(rotate_add_chain(c, s, xa, xb, bc, gs, gk_fold, nrot, batch, w.p));
    CG_TRY(do_mul(c, s, bc, kcols, d3, batch, 1, w.p, 0));
    const int rows = 3 * c->k;
    CG_LAUNCH_PW(KID_SUM_GROUPS, LB * rows * (batch + heads), (double)batch, sum_groups_kernel, pw_blocks(c, (size_t)heads * rows),
                 d3, y, (int)heads, (int)d2, rows, c->dc);
    return do_relin(c, s, y, rlk, out, heads, w.p);
}

extern "C" int cg_decode_context_outer(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *vcols,
                                       uint32_t heads, uint32_t d2, const void *rlk, const void *const *gk_all,
                                       uint64_t *out, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({a, vcols, rlk, out, ws}) && gk_all && heads >= 1 && d2 >= 1);
    const uint32_t batch = heads * d2;
    CG_REQUIRE(batch_ok(batch));
    int nrot = 0;
    uint32_t gs[20];
    for (uint32_t sh = 1; sh <= (uint32_t)c->N / 4; sh <<= 1) gs[nrot++] = pow3_mod(sh, 2u * c->N);
    gs[nrot++] = 2u * c->N - 1;
    for (int i = 0; i < nrot; i++) CG_REQUIRE(gk_all[i] && aligned16(gk_all[i]));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Bump w = bump(c, ws);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    uint64_t *xa = w.take<uint64_t>((size_t)2 * c->k * batch), *xb = w.take<uint64_t>((size_t)2 * c->k * batch);
    CG_TRY(do_mul(c, s, a, vcols, d3, batch, d2, w.p, 0));
    CG_TRY(do_relin(c, s, d3, rlk, xa, batch, w.p));
    return rotate_add_chain(c, s, xa, xb, out, gs, gk_all, nrot, batch, w.p);
}

// kp[h][sigma*H + r] (m = 2H units per head): r = 0 copies of the source, K_r = rotate(K_{r-1}, 3^d2)
// sequentially for all heads at once, then the row-swapped copies (sigma = 1)
static int rotated_copies(cg_ctx *c, hipStream_t s, const uint64_t *src, uint32_t heads, uint32_t d2,
                          const void *gk_blk, const void *gk_swap, uint64_t *kp, void *ws)
{
    const uint32_t m = (uint32_t)c->N / d2, H = m / 2;
    const size_t ct2 = (size_t)2 * c->k * c->N;
    for (uint32_t h = 0; h < heads; h++)
        CG_HIP(hipMemcpyAsync(kp + (size_t)h * m * ct2, src + (size_t)h * ct2, ct2 * 8, hipMemcpyDeviceToDevice, s));
    const uint32_t g_blk = pow3_mod(d2, 2u * c->N), g_swap = 2u * c->N - 1;
    for (uint32_t r = 1; r < H; r++)
        CG_TRY(do_rotate(c, s, kp + (size_t)(r - 1) * ct2, g_blk, gk_blk, kp + (size_t)r * ct2, heads, 0, ws,
                         (size_t)m * ct2, (size_t)m * ct2));
    for (uint32_t h = 0; h < heads; h++)
        CG_TRY(do_rotate(c, s, kp + (size_t)h * m * ct2, g_swap, gk_swap, kp + ((size_t)h * m + H) * ct2, H, 0, ws));
    return CG_OK;
}

// The same m copies per head, every one rotated out of the source itself as one series of hoisted
// rotations: unit sigma*H + r by 3^(d2 r), times 2N-1 for sigma = 1 (keys gk_copies[unit - 1])
static int rotated_copies_hoisted(cg_ctx *c, hipStream_t s, const uint64_t *src, uint32_t heads, uint32_t d2,
                                  const void *const *gk_copies, uint64_t *kp, void *ws)
{
    const uint32_t m = (uint32_t)c->N / d2, H = m / 2, two_n = 2u * c->N;
    const size_t ct2 = (size_t)2 * c->k * c->N;
    for (uint32_t h = 0; h < heads; h++)
        CG_HIP(hipMemcpyAsync(kp + (size_t)h * m * ct2, src + (size_t)h * ct2, ct2 * 8, hipMemcpyDeviceToDevice, s));
    std::vector<uint32_t> gs(m - 1);
    for (uint32_t u = 1; u < m; u++) {
        const uint64_t g = pow3_mod(d2 * (u % H), two_n);
        gs[u - 1] = (uint32_t)(u >= H ? g * (two_n - 1) % two_n : g);
    }
    return do_rotate_hoisted(c, s, src, ct2, m - 1, gs.data(), gk_copies, kp + ct2, m, heads, ws);
}

// gk_copies != null: the copies of K come from hoisted rotations (gk_blk / gk_swap are then not used)
static int prefill_qk_impl(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kk, uint32_t heads, uint32_t d2,
                           const void *rlk, const void *const *gk_fold, const void *gk_blk, const void *gk_swap,
                           const void *const *gk_copies, uint64_t *out, void *ws, uint32_t fold_w = 0)
{
    CG_REQUIRE(c && ptrs_ok({q, kk, rlk, out, ws}) && gk_fold && heads >= 1 && pow2_d(c, d2));
    const uint32_t m = (uint32_t)c->N / d2, batch = heads * m;
    CG_REQUIRE(batch_ok(batch));
    if (gk_copies) {
        for (uint32_t u = 1; u < m; u++) CG_REQUIRE(gk_copies[u - 1] && aligned16(gk_copies[u - 1]));
    } else {
        CG_REQUIRE(ptrs_ok({gk_blk, gk_swap}));
    }
    uint32_t gs[20];
    const int nrot = fold_generators(c, d2, gs);
    FoldRounds R;
    if (fold_w) {
        CG_REQUIRE(fold_rounds(c, gs, nrot, fold_w, R) && fold_keys_ok(R, gk_fold));
    } else {
        for (int i = 0; i < nrot; i++) CG_REQUIRE(gk_fold[i] && aligned16(gk_fold[i]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // kp[h][sigma*H + r]: rotated copies of K, one ciphertext per output unit
    Bump w = bump(c, ws);
    uint64_t *kp = w.take<uint64_t>((size_t)2 * c->k * batch);
    uint64_t *xb = w.take<uint64_t>((size_t)2 * c->k * batch);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    if (gk_copies) CG_TRY(rotated_copies_hoisted(c, s, kk, heads, d2, gk_copies, kp, w.p));
    else CG_TRY(rotated_copies(c, s, kk, heads, d2, gk_blk, gk_swap, kp, w.p));
    // all heads x m products at once
    CG_TRY(do_mul(c, s, q, kp, d3, batch, m, w.p, 0));
    CG_TRY(do_relin(c, s, d3, rlk, kp, batch, w.p));   // the rotated keys are consumed: reuse as x0
    if (fold_w) return fold_chain(c, s, kp, xb, out, R, gk_fold, batch, w.p);
    return rotate_add_chain(c, s, kp, xb, out, gs, gk_fold, nrot, batch, w.p);
}
extern "C" int cg_prefill_qk(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kk, uint32_t heads,
                             uint32_t d2, const void *rlk, const void *const *gk_fold, const void *gk_blk,
                             const void *gk_swap, uint64_t *out, void *ws)
{
    return prefill_qk_impl(c, stream, q, kk, heads, d2, rlk, gk_fold, gk_blk, gk_swap, nullptr, out, ws);
}
extern "C" int cg_prefill_qk_hoisted(cg_ctx *c, void *stream, const uint64_t *q, const uint64_t *kk, uint32_t heads,
                                     uint32_t d2, uint32_t fold_round_bits, const void *rlk,
                                     const void *const *gk_fold, const void *const *gk_copies, uint64_t *out, void *ws)
{
    CG_REQUIRE(gk_copies);
    return prefill_qk_impl(c, stream, q, kk, heads, d2, rlk, gk_fold, nullptr, nullptr, gk_copies, out, ws,
                           fold_round_bits);
}

static int prefill_av_impl(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *v, uint32_t heads, uint32_t d2,
                           const void *rlk, const void *gk_blk, const void *gk_swap, const void *const *gk_copies,
                           uint64_t *out, void *ws, bool sum_first = false)
{
    CG_REQUIRE(c && ptrs_ok({a, v, rlk, out, ws}) && heads >= 1 && pow2_d(c, d2));
    const uint32_t m = (uint32_t)c->N / d2, batch = heads * m;
    CG_REQUIRE(batch_ok(batch));
    if (gk_copies) {
        for (uint32_t u = 1; u < m; u++) CG_REQUIRE(gk_copies[u - 1] && aligned16(gk_copies[u - 1]));
    } else {
        CG_REQUIRE(ptrs_ok({gk_blk, gk_swap}));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    Bump w = bump(c, ws);
    uint64_t *vp = w.take<uint64_t>((size_t)2 * c->k * batch);
    uint64_t *d3 = w.take<uint64_t>((size_t)3 * c->k * batch);
    uint64_t *y = w.take<uint64_t>((size_t)3 * c->k * heads);
    if (gk_copies) CG_TRY(rotated_copies_hoisted(c, s, v, heads, d2, gk_copies, vp, w.p));
    else CG_TRY(rotated_copies(c, s, v, heads, d2, gk_blk, gk_swap, vp, w.p));
    if (sum_first) {
        CG_TRY(do_mul(c, s, a, vp, y, batch, 1, w.p, 0, 0, 0, nullptr, m));
    } else {
        CG_TRY(do_mul(c, s, a, vp, d3, batch, 1, w.p, 0));
        const int rows = 3 * c->k;
        CG_LAUNCH_PW(KID_SUM_GROUPS, (double)limb_bytes(c) * rows * (batch + heads), (double)batch, sum_groups_kernel,
                     pw_blocks(c, (size_t)heads * rows), d3, y, (int)heads, (int)m, rows, c->dc);
    }
    return do_relin(c, s, y, rlk, out, heads, w.p);
}
extern "C" int cg_prefill_av(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *v, uint32_t heads,
                             uint32_t d2, const void *rlk, const void *gk_blk, const void *gk_swap, uint64_t *out,
                             void *ws)
{
    return prefill_av_impl(c, stream, a, v, heads, d2, rlk, gk_blk, gk_swap, nullptr, out, ws);
}
extern "C" int cg_prefill_av_hoisted(cg_ctx *c, void *stream, const uint64_t *a, const uint64_t *v, uint32_t heads,
                                     uint32_t d2, int sum_before_scaling, const void *rlk,
                                     const void *const *gk_copies, uint64_t *out, void *ws)
{
    CG_REQUIRE(gk_copies && (sum_before_scaling == 0 || sum_before_scaling == 1));
    return prefill_av_impl(c, stream, a, v, heads, d2, rlk, nullptr, nullptr, gk_copies, out, ws,
                           sum_before_scaling != 0);
}

extern "C" int cg_prefill_repack(cg_ctx *c, void *stream, const uint64_t *x, uint32_t heads, uint32_t d2,
                                 const void *mask0, const void *const *gk_right, uint64_t *out, void *ws)
{
    CG_REQUIRE(c && ptrs_ok({x, mask0, out, ws}) && gk_right && heads >= 1 && pow2_d(c, d2));
    const uint32_t m = (uint32_t)c->N / d2, H = m / 2, batch = heads * m;
    CG_REQUIRE(batch_ok(batch));
    const uint32_t wdt = H < d2 ? H : d2;        // diagonals packed into one output
    const uint32_t n_out = batch / wdt;
    int levels = 0;
    for (uint32_t sh = 1; sh < wdt; sh <<= 1) {
        CG_REQUIRE(gk_right[levels] && aligned16(gk_right[levels]));
        levels++;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t ct2 = (size_t)2 * c->k * c->N;
    const double LB = (double)limb_bytes(c);
    Bump w = bump(c, ws);
    uint64_t *y = w.take<uint64_t>((size_t)2 * c->k * batch);
    double *f = w.take<double>((size_t)2 * c->k * batch);
    // y[u] = x[u] * mask0 (keeps slot 0 of every block)
    const size_t rows = (size_t)batch * 2 * c->k;
    CG_TRY(launch_fwd(c, s, rows, LdRowsU64{x, nullptr, c->k, c->logn}, StF64{f, c->logn}, KID_FWD_ROWS,
                      LB * 2.0 * rows));
    CG_TRY(launch_inv(c, s, rows, LdInvMulPlain{f, static_cast<const double *>(mask0), 1, 1 << 30, 0, 0, c->logn},
                      StInvU64{y, c->logn}, KID_INV_MULPLAIN, LB * (2.0 * rows + c->k)));
    // pairwise tree inside every group of wdt consecutive units: at level l (shift 2^l)
    // y[j 2^(l+1)] += rotate_right(y[j 2^(l+1) + 2^l], 2^l); rotate right by sh = Galois 3^(N/2 - sh)
    for (int l = 0; l < levels; l++) {
        const uint32_t sh = 1u << l;
        const size_t stride = (size_t)2 * sh * ct2;
        CG_TRY(do_rotate(c, s, y + (size_t)sh * ct2, pow3_mod((uint32_t)c->N / 2 - sh, 2u * c->N), gk_right[l], y,
                         batch / (2 * sh), 1, w.p, stride, stride, y, stride));
    }
    // gather the group leaders
    for (uint32_t o = 0; o < n_out; o++)
        CG_HIP(hipMemcpyAsync(out + (size_t)o * ct2, y + (size_t)o * wdt * ct2, ct2 * 8, hipMemcpyDeviceToDevice, s));
    return CG_OK;
}

// One token times `units` plaintext matrices (the decode step's ciphertext-plaintext vector-matrix
// product): rotated copies of the token by a doubling tree, the products with the diagonals summed
// on the way into one inverse transform per unit, then the sum over residue classes modulo d2.
// gk_copies != null: the rotated copies of the token are a series of hoisted rotations of the token
// itself (copy c by 3^c, key gk_copies[c - 1]) instead of the doubling tree over gk_shift
static int cpvm_impl(cg_ctx *c, void *stream, const uint64_t *x, const void *diags, uint32_t units, uint32_t n_diag,
                     uint32_t d2, const void *const *gk_shift, const void *const *gk_copies,
                     const void *const *gk_block, uint64_t *out, void *ws, uint32_t block_w = 0)
{
    CG_REQUIRE(c && ptrs_ok({x, diags, out, ws}) && gk_block && batch_ok(units) && pow2_d(c, d2));
    CG_REQUIRE(n_diag >= 1 && n_diag <= 64 && (n_diag & (n_diag - 1)) == 0 && n_diag <= d2);
    CG_REQUIRE(n_diag == 1 || gk_shift || gk_copies);
    CG_REQUIRE(!overlap(x, 2 * (size_t)c->k * limb_bytes(c), out, 2 * (size_t)c->k * limb_bytes(c) * units));
    if (gk_copies) {
        for (uint32_t cc = 1; cc < n_diag; cc++) CG_REQUIRE(gk_copies[cc - 1] && aligned16(gk_copies[cc - 1]));
    } else {
        int levels = 0;
        for (uint32_t sh = 1; sh < n_diag; sh <<= 1, levels++) CG_REQUIRE(gk_shift[levels] && aligned16(gk_shift[levels]));
    }
    uint32_t gs[20];
    const int nrot = block_generators(c, d2, gs);
    FoldRounds R;
    if (block_w) {
        CG_REQUIRE(fold_rounds(c, gs, nrot, block_w, R) && fold_keys_ok(R, gk_block));
    } else {
        for (int i = 0; i < nrot; i++) CG_REQUIRE(gk_block[i] && aligned16(gk_block[i]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t ct2 = (size_t)2 * c->k * c->N;
    const double LB = (double)limb_bytes(c);
    Bump w = bump(c, ws);
    uint64_t *copies = w.take<uint64_t>((size_t)2 * c->k * n_diag);
    double *f = w.take<double>((size_t)2 * c->k * n_diag);
    uint64_t *xa = w.take<uint64_t>((size_t)2 * c->k * units), *xb = w.take<uint64_t>((size_t)2 * c->k * units);
    CG_HIP(hipMemcpyAsync(copies, x, ct2 * 8, hipMemcpyDeviceToDevice, s));
    if (gk_copies && n_diag > 1) {
        uint32_t cg[64];
        for (uint32_t cc = 1; cc < n_diag; cc++) cg[cc - 1] = pow3_mod(cc, 2u * c->N);
        CG_TRY(do_rotate_hoisted(c, s, x, ct2, n_diag - 1, cg, gk_copies, copies + ct2, n_diag, 1, w.p));
    } else {
        // copy 2^l + i = copy i rotated left by 2^l
        for (uint32_t sh = 1, l = 0; sh < n_diag; sh <<= 1, l++)
            CG_TRY(do_rotate(c, s, copies, pow3_mod(sh, 2u * c->N), gk_shift[l], copies + (size_t)sh * ct2, sh, 0, w.p));
    }
    const size_t crows = (size_t)n_diag * 2 * c->k, rows = (size_t)units * 2 * c->k;
    CG_TRY(launch_fwd(c, s, crows, LdRowsU64{copies, nullptr, c->k, c->logn}, StF64Red{f, c->logn}, KID_FWD_ROWS,
                      LB * 2.0 * crows));
    CG_TRY(launch_inv(c, s, rows, LdInvPlainSum{f, static_cast<const double *>(diags), (int)n_diag, c->logn},
                      StInvU64{xa, c->logn}, KID_INV_MULPLAIN,
                      LB * (crows + (double)units * n_diag * c->k + rows)));
    if (block_w) return fold_chain(c, s, xa, xb, out, R, gk_block, units, w.p);
    return rotate_add_chain(c, s, xa, xb, out, gs, gk_block, nrot, units, w.p);
}
extern "C" int cg_cpvm(cg_ctx *c, void *stream, const uint64_t *x, const void *diags, uint32_t units,
                       uint32_t n_diag, uint32_t d2, const void *const *gk_shift, const void *const *gk_block,
                       uint64_t *out, void *ws)
{
    return cpvm_impl(c, stream, x, diags, units, n_diag, d2, gk_shift, nullptr, gk_block, out, ws);
}
extern "C" int cg_cpvm_hoisted(cg_ctx *c, void *stream, const uint64_t *x, const void *diags, uint32_t units,
                               uint32_t n_diag, uint32_t d2, uint32_t block_round_bits,
                               const void *const *gk_copies, const void *const *gk_block, uint64_t *out, void *ws)
{
    CG_REQUIRE(n_diag == 1 || gk_copies);
    return cpvm_impl(c, stream, x, diags, units, n_diag, d2, nullptr, gk_copies, gk_block, out, ws, block_round_bits);
}

// Every transform-kernel instantiation this context can launch, at a batch below and one above the
// number of compute units (the forward plan depends on it).  Runs with c->dry set: the launch
// helpers look the kernel's occupancy up, record it and return before launching, so the dummy
// addresses are never dereferenced.
static int warm_launch_table(cg_ctx *c)
{
    hipStream_t s = nullptr;
    uint64_t *u = reinterpret_cast<uint64_t *>(uintptr_t(1) << 20);
    double *f = reinterpret_cast<double *>(uintptr_t(1) << 20);
    const double LB = 0.0;
    for (uint32_t batch : {1u, 4096u}) {
        CG_TRY(do_mul(c, s, u, u, u, batch, 1, f, 0));
        CG_TRY(do_mul(c, s, u, u, u, batch, 1, f, 0, 0, 0, nullptr, 1));
        CG_TRY(do_keyswitch(c, s, u, 0, 0, f, u, 0, u, 0, 0, 0, batch, f));
        CG_TRY(do_keyswitch(c, s, u, 0, 3, f, u, 0, u, 0, 3, 1, batch, f));
        {
            const uint32_t gs1[1] = {3};
            const void *const keys1[1] = {f};
            CG_TRY(do_rotate_hoisted(c, s, u, 0, 1, gs1, keys1, u, 1, batch, f));
            CG_TRY(do_rotate_sum(c, s, u, 0, 1, gs1, keys1, u, 0, batch, f));
        }
        const size_t rows = (size_t)batch * 2 * c->k;
        const LdRowsU64 ld{u, nullptr, c->k, c->logn};
        CG_TRY(launch_fwd(c, s, rows, ld, StU64{u, c->logn}, KID_FWD_ROWS, LB));
        CG_TRY(launch_fwd(c, s, rows, ld, StF64{f, c->logn}, KID_FWD_ROWS, LB));
        CG_TRY(launch_fwd(c, s, rows, ld, StF64Red{f, c->logn}, KID_FWD_ROWS, LB));
        CG_TRY(launch_fwd(c, s, rows, LdPlain{u, c->logn}, StF64Red{f, c->logn}, KID_FWD_PLAIN, LB));
        CG_TRY(launch_inv(c, s, rows, LdInvU64{u, nullptr, c->k, c->logn}, StInvU64{u, c->logn}, KID_INV_U64, LB));
        const LdInvMulPlain mp{f, f, 1, 1, 0, 0, c->logn};
        CG_TRY(launch_inv(c, s, rows, mp, StInvU64{u, c->logn}, KID_INV_MULPLAIN, LB));
        CG_TRY(launch_inv(c, s, rows, mp, StInvAppend{u, 0, 1, c->logn}, KID_INV_MULPLAIN, LB));
        CG_TRY(launch_inv(c, s, rows, LdInvPlainSum{f, f, 1, c->logn}, StInvU64{u, c->logn}, KID_INV_MULPLAIN, LB));
    }
    return CG_OK;
}

extern "C" int cg_profile_begin(cg_ctx *c, uint32_t max_launches)
{
    CG_REQUIRE(c && max_launches >= 1 && max_launches <= (1u << 20) && !c->prof_on);
    if (c->prof_cap < max_launches) {
        for (uint32_t i = 0; i < 2 * c->prof_cap; i++) (void)hipEventDestroy(c->prof_ev[i]);
        delete[] c->prof_ev; delete[] c->prof_id; delete[] c->prof_bytes; delete[] c->prof_items;
        c->prof_cap = 0;
        c->prof_ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_launches];
        c->prof_id = new (std::nothrow) uint8_t[max_launches];
        c->prof_bytes = new (std::nothrow) double[max_launches];
        c->prof_items = new (std::nothrow) double[max_launches];
        if (!c->prof_ev || !c->prof_id || !c->prof_bytes || !c->prof_items) return CG_ENOMEM;
        for (uint32_t i = 0; i < 2 * max_launches; i++) CG_HIP(hipEventCreate(&c->prof_ev[i]));
        c->prof_cap = max_launches;
    }
    c->prof_n = 0;
    c->prof_on = true;
    return CG_OK;
}

extern "C" int cg_profile_end(cg_ctx *c, cg_kernel_stat *stats, uint32_t cap, uint32_t *n_out)
{
    CG_REQUIRE(c && stats && n_out && c->prof_on);
    c->prof_on = false;
    cg_kernel_stat acc[KID_COUNT];
    memset(acc, 0, sizeof(acc));
    for (uint32_t i = 0; i < c->prof_n; i++) {
        CG_HIP(hipEventSynchronize(c->prof_ev[2 * i + 1]));
        float ms = 0.f;
        CG_HIP(hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
        cg_kernel_stat &k = acc[c->prof_id[i]];
        k.launches++;
        k.total_ms += ms;
        k.algo_bytes += c->prof_bytes[i];
        k.work_items += c->prof_items[i];
    }
    uint32_t n = 0;
    for (int id = 0; id < KID_COUNT; id++)
        if (acc[id].launches && n < cap) {
            acc[id].kernel_id = (uint32_t)id;
            stats[n++] = acc[id];
        }
    *n_out = n;
    return CG_OK;
}

extern "C" const char *cg_kernel_name(uint32_t id) { return id < KID_COUNT ? kKernelNames[id] : "?"; }

extern "C" int cg_bench_exchange(cg_ctx *c, void *stream, int kind, uint32_t n_blocks, uint32_t iters, double *out)
{
    CG_REQUIRE(c && ptrs_ok({out}) && (kind == 0 || kind == 1) && n_blocks >= 1 && n_blocks <= (1u << 16));
    return launch_kernel(bench_exchange_kernel, dim3(n_blocks), dim3(1024), static_cast<hipStream_t>(stream), kind,
                         iters, out);
}

extern "C" int cg_bench_modmul(cg_ctx *c, void *stream, int kind, uint32_t n_lanes, uint32_t iters, uint64_t *out)
{
    CG_REQUIRE(c && ptrs_ok({out}) && (kind == 0 || kind == 1) && n_lanes >= 1 && c->pr[0] > (1ull << 49));
    ModI mi{c->pr[0], (uint64_t)((((u128)1) << 100) / c->pr[0])};
    return launch_kernel(bench_modmul_kernel, dim3((n_lanes + PW_THREADS - 1) / PW_THREADS), dim3(PW_THREADS),
                         static_cast<hipStream_t>(stream), kind, n_lanes, iters, out, c->hc.mod[0], mi);
}
