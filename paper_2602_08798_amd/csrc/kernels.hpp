// Device kernels (gfx950).  One workgroup transforms one residue row ("limb")
// that stays in LDS for the whole transform; everything else is pointwise.
#pragma once
#include <hip/hip_runtime.h>
#include "tables.hpp"

namespace cg {

// ---------------------------------------------------------------------------
// Transform plan.  A row of N = 2^LOGN residues is transformed by one workgroup
// of N / E threads; each thread keeps E elements in registers and a pass runs
// R butterfly stages on them between two LDS exchanges.  The first NC passes pair
// elements owned by different waves (workgroup barrier); after them every wave
// owns one contiguous chunk of 64 * E elements and all remaining stages stay
// inside it, so those passes only need wave-level ordering.
//   N = 8192: forward kernels run E = 16 (512 threads, registers capped at 128 so that two
//   workgroups share a compute unit and cover each other's loads; no register prefetch), which
//   measured 5-10 % faster than E = 8; the inverse kernels keep E = 8 (their fused loaders spill
//   at 128 registers).  E = 16 is the only choice at N = 16384 (1024 threads).
// ---------------------------------------------------------------------------
template <int LOGN, int E> struct Plan;
template <> struct Plan<14, 16> { static constexpr int NP = 4, NC = 1; static constexpr int R[5] = {4, 4, 3, 3, 0}; };
template <> struct Plan<12, 8> { static constexpr int NP = 4, NC = 1; static constexpr int R[5] = {3, 3, 3, 3, 0}; };
template <> struct Plan<13, 8> { static constexpr int NP = 5, NC = 2; static constexpr int R[5] = {3, 3, 3, 3, 1}; };
template <> struct Plan<13, 16> { static constexpr int NP = 4, NC = 1; static constexpr int R[5] = {4, 3, 3, 3, 0}; };
// The next row is prefetched into registers where that helps: not with two workgroups on a compute
// unit (each covers the other's load latency), and not at N = 16384, where the prefetched words
// push the 128-register budget of a 1024-thread workgroup into spilling (measured: C5 step
// 4.58 -> 4.29 ms without).
template <int LOGN, int E> constexpr bool prefetch_rows() { return LOGN <= 12 || (LOGN == 13 && E == 8); }
// waves per SIMD the register allocation must leave room for: the workgroup's own, or, for rows of
// 8192 on 512 threads, twice that, so that two workgroups share a compute unit (2 x 72 KiB of LDS)
template <int LOGN, int E> constexpr int min_waves() { return (LOGN == 13 && E == 16) ? 4 : ((1 << LOGN) / E) / 256; }

constexpr int ilog2c(int x) { return x <= 1 ? 0 : 1 + ilog2c(x / 2); }
template <int E> constexpr int chunk_log() { return 6 + ilog2c(E); }

template <int LOGN, int E, int PASS> constexpr int stage_start()
{
    int s = 0;
    for (int i = 0; i < PASS; i++) s += Plan<LOGN, E>::R[i];
    return s;
}

// group index of a thread in pass PASS (g-th group of the thread)
template <int LOGN, int E, int PASS> __device__ __forceinline__ int group_index(int tid, int g)
{
    constexpr int R = Plan<LOGN, E>::R[PASS];
    if (PASS < Plan<LOGN, E>::NC) return tid + g * ((1 << LOGN) / E);
    int lane = tid & 63;
    // a radix-2 pass works on pairs of neighbours, 16 bytes per lane: which pair a lane takes is
    // permuted as in chunk_elem, for the same reason (LDS banks)
    if (R == 1) lane = (lane & 7) | (((lane >> 4) & 3) << 3) | (((lane >> 3) & 1) << 5);
    return ((tid >> 6) << (chunk_log<E>() - R)) + lane + 64 * g;
}
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would drain the next row's prefetch at each
// barrier; threads of these kernels exchange data through LDS alone.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// compiler-level ordering between LDS writes and reads of the same wave (the LDS pipeline
// itself executes one wave's operations in order)
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
}

// Forward stage bound: |out| <= 1.1875 |in| + 0.5 (in units of p).  Values must
// stay below 8p = 2^53.
constexpr double fwd_grow(double b, int stages)
{
    for (int i = 0; i < stages; i++) b = 1.1875 * b + 0.5;
    return b;
}
// Decide at compile time which forward passes start with a reduction.
template <int LOGN, int E, int PASS> struct FwdBound {
    static constexpr double in_prev = FwdBound<LOGN, E, PASS - 1>::out;
    static constexpr bool reduce = fwd_grow(in_prev, Plan<LOGN, E>::R[PASS]) > 7.5;
    static constexpr double out = fwd_grow(reduce ? 0.51 : in_prev, Plan<LOGN, E>::R[PASS]);
};
template <int LOGN, int E> struct FwdBound<LOGN, E, 0> {
    static constexpr bool reduce = false;                       // loaders deliver |x| <= p
    static constexpr double out = fwd_grow(1.0, Plan<LOGN, E>::R[0]);
};

__device__ __forceinline__ void bfly_fwd(double &a, double &b, double w, const ModD m)
{
    const double t = mulmod(b, w, m);
    b = a - t;
    a = a + t;
}
__device__ __forceinline__ void bfly_inv(double &a, double &b, double w, const ModD m)
{
    const double d = a - b;
    a = a + b;
    b = mulmod(d, w, m);
}

// ---------------------------------------------------------------------------
// twiddles of one pass, fetched into registers ahead of the synchronisation
// that precedes the pass: slot (g, (1<<u) - 1 + j) holds the factor of stage
// S0+u for the j-th sub-block of group g
// ---------------------------------------------------------------------------
constexpr int TWREGS = 16;

// LDS layout: one pad double after every 8, so that a thread owning 8 (or 16)
// consecutive elements is 9 doubles away from its neighbour lane and the
// stride-1 passes are bank-conflict free.  For the index patterns used here
// (base + (c << L), base = (hi << (L+R)) | lo with lo < 2^L) the pad of the sum
// is the sum of the pads -- with L >= 3 the element part is a multiple of 8,
// otherwise it never carries out of the group's aligned span -- so the
// per-element part folds into instruction offsets.
__device__ __forceinline__ constexpr int pad(int idx) { return idx + (idx >> 3); }
template <int LOGN> constexpr int lds_doubles() { return (1 << LOGN) + (1 << (LOGN - 3)); }

template <int LOGN, int E, int PASS, bool HI_ZERO>
__device__ __forceinline__ void load_tw(const double *__restrict__ tw, int tid, double *twr)
{
    using P = Plan<LOGN, E>;
    constexpr int R = P::R[PASS];
    constexpr int S0 = stage_start<LOGN, E, PASS>();
    constexpr int L = LOGN - S0 - R;
    constexpr int G = E >> R;
    constexpr int PER = (1 << R) - 1;
    static_assert(G * PER <= TWREGS, "twiddle register file too small");
#pragma unroll
    for (int g = 0; g < G; g++) {
        int hi = HI_ZERO ? 0 : (group_index<LOGN, E, PASS>(tid, g) >> L);
        // with L >= 6 all 64 lanes of a wave share hi: say so, and the factors come in through
        // the scalar cache instead of one vector load per lane
        if (!HI_ZERO && PASS > 0 && L >= 6) hi = __builtin_amdgcn_readfirstlane(hi);
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
            for (int j = 0; j < (1 << u); j++)
                twr[g * PER + (1 << u) - 1 + j] = tw[(1 << (S0 + u)) + (hi << u) + j];
    }
}

// ---------------------------------------------------------------------------
// Workgroups are handed to the 8 XCDs round-robin (physical index p runs on XCD p % 8), each
// with its own L2.  Rows that read the same operand are neighbours in logical order, in groups
// of S (the loader's share()); this bijection on [0, nwg) gives every XCD whole groups, so the
// operand comes from HBM once and from that XCD's L2 afterwards: within each full block of 8*S
// physical indices, XCD x takes the logical rows block*8S + x*S ... + S-1.  (Grids are multiples
// of 8 whenever a workgroup walks over more than one row.)
// ---------------------------------------------------------------------------
__device__ __forceinline__ int xcd_row(int p, int nwg, int S)
{
    const int blk = 8 * S;
    const int full = nwg - nwg % blk;
    if (S == 1 || p >= full) return p;
    const int b = p / blk, w = p - b * blk;
    return b * blk + (w & 7) * S + (w >> 3);
}

// ---------------------------------------------------------------------------
// The transform kernels are persistent: a workgroup walks over rows
// wg = blockIdx.x, blockIdx.x + gridDim.x, ... and, while it transforms one row,
// the raw words of its next row are already on their way into registers.
//
// Loader interface (LD):
//   kRaw                       64-bit words fetched per element
//   kPrefetch                  fetch the next row during the current one (else fetch in slices at use)
//   kScatter                   forward only: elements are placed into LDS at place(idx) before pass 0
//   prime(wg, C)               prime index of row wg
//   dst_limb(wg, C)            forward only: destination row
//   fetch(wg, idx, C, raw)     issue the loads of element idx (no arithmetic on the loaded words)
//   finish(raw, wg, idx, m, C) element value, |x| <= p (forward) or < 8p (inverse)
//
// Element ownership: CHUNKED = false: element it of a thread is tid + it * T
// (pass 0); CHUNKED = true: (wave << chunk_log) + lane + 64 * it (the wave's chunk).
// Both put consecutive lanes on consecutive addresses.
// ---------------------------------------------------------------------------
// element `it` of a thread in the chunked ownership: a lane takes pairs of neighbouring elements of
// its wave's chunk, so that every operand comes in (and every result goes out) 16 bytes per lane.
// Which pair: lane bits 0-2 give pair bits 0-2, lane bit 3 pair bit 5, lane bits 4-5 pair bits 3-4,
// the iteration the bits above.  Eight consecutive lanes then cover one 128-byte line in memory,
// and in the padded LDS row (position = index + index / 8) any sixteen consecutive lanes land on
// sixteen different 8-byte banks: pair u = a + 4 b sits at 2 a + 9 b, and b in {0, 1, 8, 9} gives
// offsets 0, 9, 8, 1 modulo 16.  With lane l simply taking pair l, lanes l and l + 8 collide.
template <int E> __device__ __forceinline__ int chunk_elem(int tid, int it)
{
    const int lane = tid & 63;
    const int u = (lane & 7) | (((lane >> 4) & 3) << 3) | (((lane >> 3) & 1) << 5);
    return ((tid >> 6) << chunk_log<E>()) + 2 * u + (it & 1) + 128 * (it >> 1);
}

template <int LOGN, int E, bool CHUNKED, class LD>
__device__ __forceinline__ void fetch_row(const LD &ld, int wg, int tid, const DevConst *C,
                                          uint64_t (&raw)[E][LD::kRaw])
{
    constexpr int T = (1 << LOGN) / E;
#pragma unroll
    for (int it = 0; it < E; it++) ld.fetch(wg, CHUNKED ? chunk_elem<E>(tid, it) : tid + it * T, C, raw[it]);
}

// Loaders whose element is a sum over several rounds of fetches (ld.rounds() of them, each with
// ld.fetch_round / ld.finish, the partial sums joined by ld.join) are marked here.
template <class LD> struct ld_rounds { static constexpr bool value = false; };

// Loaders that do not prefetch fetch and finish a row in slices, so that at most about 32 raw
// words are live per thread however many words an element needs.
template <int LOGN, int E, bool CHUNKED, class LD, class F>
__device__ __forceinline__ void load_row_now(const LD &ld, int wg, int tid, const ModD m, const DevConst *C, F &&sink)
{
    constexpr int T = (1 << LOGN) / E;
    constexpr int CH0 = LD::kRaw <= 2 ? 16 : (LD::kRaw <= 4 ? (E >= 16 && CHUNKED ? 4 : 8) : (E >= 16 && CHUNKED ? 2 : 4));
    constexpr int CH = CH0 < E ? CH0 : E;
    auto at = [&](int it) { return CHUNKED ? chunk_elem<E>(tid, it) : tid + it * T; };
    if constexpr (ld_rounds<LD>::value) {
        const int nr = ld.rounds();
#pragma unroll
        for (int c0 = 0; c0 < E; c0 += CH) {
            double sum[CH];
#pragma unroll
            for (int i = 0; i < CH; i++) sum[i] = 0.0;
            for (int r = 0; r < nr; r++) {
                uint64_t rw[CH][LD::kRaw];
#pragma unroll
                for (int i = 0; i < CH; i++) ld.fetch_round(wg, at(c0 + i), r, C, rw[i]);
#pragma unroll
                for (int i = 0; i < CH; i++) sum[i] = ld.join(sum[i], ld.finish(rw[i], wg, at(c0 + i), m, C), m);
            }
#pragma unroll
            for (int i = 0; i < CH; i++) sink(c0 + i, at(c0 + i), sum[i]);
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
#pragma unroll
    for (int c0 = 0; c0 < E; c0 += CH) {
        uint64_t rw[CH][LD::kRaw];
#pragma unroll
        for (int i = 0; i < CH; i++) ld.fetch(wg, at(c0 + i), C, rw[i]);
#pragma unroll
        for (int i = 0; i < CH; i++) sink(c0 + i, at(c0 + i), ld.finish(rw[i], wg, at(c0 + i), m, C));
        // keep the slices apart: hoisting the next slice's loads above this one's arithmetic
        // would bring back the register pressure the slicing is there to avoid
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ---------------------------------------------------------------------------
// forward transform
// ---------------------------------------------------------------------------
template <int LOGN, int E, int PASS, bool FROM_REGS, class ST>
__device__ __forceinline__ void fwd_pass(double *lds, const double *in, const ST &st, int tid,
                                         const double *__restrict__ tw, const double *twr, double *twr_next,
                                         const ModD m, int dst_limb)
{
    using P = Plan<LOGN, E>;
    constexpr int R = P::R[PASS];
    constexpr int S0 = stage_start<LOGN, E, PASS>();
    constexpr int L = LOGN - S0 - R;          // index bits below this pass's R bits
    constexpr int G = E >> R;                 // independent radix-2^R groups per thread
    constexpr int PER = (1 << R) - 1;
    constexpr bool first = PASS == 0, last = PASS == P::NP - 1;
    constexpr bool cross = PASS < P::NC;      // pairs elements owned by different waves
    constexpr bool do_red = FwdBound<LOGN, E, PASS>::reduce;
    static_assert(FwdBound<LOGN, E, PASS>::out < 8.0, "lazy bound exceeds 2^53");
    static_assert(!FROM_REGS || (first && L + R == LOGN), "register input only for the first pass");
    static_assert(cross || L + R <= chunk_log<E>(), "wave-local passes must stay inside one chunk");
    static_assert(!last || !cross, "the last pass must be wave-local (chunk-wise copy-out)");
    double v[G][1 << R];
    int base[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const int gidx = group_index<LOGN, E, PASS>(tid, g);
        const int lo = gidx & ((1 << L) - 1);
        const int hi = first ? 0 : (gidx >> L);
        base[g] = (hi << (L + R)) | lo;
        const int pb = pad(base[g]);
#pragma unroll
        for (int c = 0; c < (1 << R); c++) {
            // first pass: element base + (c << L) = tid + (g + c*G) * T is fetched element g + c*G
            if (FROM_REGS) v[g][c] = in[g + c * G];
            else v[g][c] = lds[pb + pad(c << L)];
        }
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
        if (do_red) {
#pragma unroll
            for (int c = 0; c < (1 << R); c++) v[g][c] = red(v[g][c], m);
        }
#pragma unroll
        for (int u = 0; u < R; u++) {
            const int half = 1 << (R - 1 - u);
#pragma unroll
            for (int c = 0; c < (1 << R); c++) {
                if (c & half) continue;
                bfly_fwd(v[g][c], v[g][c + half], twr[g * PER + (1 << u) - 1 + (c >> (R - u))], m);
            }
        }
    }
    // fetch the next pass's factors while this pass's results drain to LDS
    if constexpr (!last) load_tw<LOGN, E, PASS + 1, false>(tw, tid, twr_next);
#pragma unroll
    for (int g = 0; g < G; g++) {
        const int pb = pad(base[g]);
#pragma unroll
        for (int c = 0; c < (1 << R); c++) lds[pb + pad(c << L)] = v[g][c];
    }
    if constexpr (cross) lds_barrier();
    else wave_sync();
    if constexpr (last) {
        // results leave through LDS so that consecutive lanes write consecutive addresses; each
        // wave copies out its own chunk
        // (a lane takes pairs of neighbouring elements: 16 bytes per lane and store)
#pragma unroll
        for (int it = 0; it < E; it++) {
            const int idx = chunk_elem<E>(tid, it);
            st.store(dst_limb, idx, lds[pad(idx)], m);
        }
    }
}

template <int LOGN, int E, class LD, class ST>
__global__ void __launch_bounds__((1 << LOGN) / E, (min_waves<LOGN, E>()))
ntt_fwd_kernel(LD ld, ST st, const double *__restrict__ tw_all, const DevConst *__restrict__ C, int nwg)
{
    __shared__ double lds[lds_doubles<LOGN>()];
    constexpr bool PF = LD::kPrefetch && prefetch_rows<LOGN, E>();
    constexpr int T = (1 << LOGN) / E;
    constexpr int NP = Plan<LOGN, E>::NP;
    const int tid = threadIdx.x;
    const int S = ld.share(C);
    int p = blockIdx.x;
    int wg = xcd_row(p, nwg, S);
    // loaders that scatter into LDS before pass 0 are free in which elements a thread brings in:
    // they use the chunked ownership; the others bring in what pass 0 works on in registers
    constexpr bool CH = LD::kScatter;
    uint64_t raw[PF ? E : 1][LD::kRaw];
    if constexpr (PF) fetch_row<LOGN, E, CH>(ld, wg, tid, C, raw);
    for (;;) {
        const int pr = ld.prime(wg, C);
        const ModD m = C->mod[pr];
        const double *tw = tw_all + ((size_t)pr << LOGN);
        const int dl = ld.dst_limb(wg, C);
        double twa[TWREGS], twb[TWREGS];
        load_tw<LOGN, E, 0, true>(tw, tid, twa);
        double in[E];
        p += (int)gridDim.x;
        const bool more = p < nwg;
        const int wg_next = more ? xcd_row(p, nwg, S) : 0;
        if constexpr (PF) {
#pragma unroll
            for (int it = 0; it < E; it++)
                in[it] = ld.finish(raw[it], wg, CH ? chunk_elem<E>(tid, it) : tid + it * T, m, C);
            if (more) fetch_row<LOGN, E, CH>(ld, wg_next, tid, C, raw);
        } else {
            load_row_now<LOGN, E, CH>(ld, wg, tid, m, C, [&](int it, int, double v) { in[it] = v; });
        }
        if constexpr (LD::kScatter) {
#pragma unroll
            for (int it = 0; it < E; it++) lds[pad(ld.place(chunk_elem<E>(tid, it), 1 << LOGN))] = in[it];
            lds_barrier();
            fwd_pass<LOGN, E, 0, false>(lds, in, st, tid, tw, twa, twb, m, dl);
        } else {
            fwd_pass<LOGN, E, 0, true>(lds, in, st, tid, tw, twa, twb, m, dl);
        }
        fwd_pass<LOGN, E, 1, false>(lds, in, st, tid, tw, twb, twa, m, dl);
        fwd_pass<LOGN, E, 2, false>(lds, in, st, tid, tw, twa, twb, m, dl);
        if constexpr (NP > 3) fwd_pass<LOGN, E, 3, false>(lds, in, st, tid, tw, twb, twa, m, dl);
        if constexpr (NP > 4) fwd_pass<LOGN, E, 4, false>(lds, in, st, tid, tw, twa, twb, m, dl);
        if (!more) break;
        wg = wg_next;
        lds_barrier();   // the copy-out reads of this row precede the next row's LDS writes
    }
}

// ---------------------------------------------------------------------------
// inverse transform (passes in reverse order; N^-1 folded into the last stage)
// ---------------------------------------------------------------------------
template <int LOGN, int E, int PASS, class ST>
__device__ __forceinline__ void inv_pass(double *lds, const ST &st, int wg, int tid,
                                         const double *__restrict__ itw, const double *twr, double *twr_next,
                                         const ModD m, int pr, const DevConst *C)
{
    using P = Plan<LOGN, E>;
    constexpr int R = P::R[PASS];
    constexpr int S0 = stage_start<LOGN, E, PASS>();
    constexpr int L = LOGN - S0 - R;
    constexpr int G = E >> R;
    constexpr int PER = (1 << R) - 1;
    constexpr bool last = PASS == 0;
    constexpr bool cross = PASS < P::NC;
    static_assert(cross || L + R <= chunk_log<E>(), "wave-local passes must stay inside one chunk");
    double v[G][1 << R];
    int base[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
        // the last pass stores straight to global memory and all its groups share their twiddles:
        // with an even number of groups a thread takes neighbouring ones (16 bytes per lane and store)
        const int gidx = (last && G % 2 == 0) ? 2 * tid + (g & 1) + 2 * ((1 << LOGN) / E) * (g >> 1)
                                              : group_index<LOGN, E, PASS>(tid, g);
        const int lo = gidx & ((1 << L) - 1);
        const int hi = last ? 0 : (gidx >> L);
        base[g] = (hi << (L + R)) | lo;
        const int pb = pad(base[g]);
#pragma unroll
        for (int c = 0; c < (1 << R); c++) v[g][c] = lds[pb + pad(c << L)];
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
        // every pass starts from |x| <= p/2: the sum path doubles per stage
#pragma unroll
        for (int c = 0; c < (1 << R); c++) v[g][c] = red(v[g][c], m);
#pragma unroll
        for (int u = R - 1; u >= 0; u--) {
            const int half = 1 << (R - 1 - u);
            if (R == 4 && u == 1) {   // after two stages of a four-stage pass: |x| <= 2p -> p/2
#pragma unroll
                for (int c = 0; c < (1 << R); c++) v[g][c] = red(v[g][c], m);
            }
#pragma unroll
            for (int c = 0; c < (1 << R); c++) {
                if (c & half) continue;
                if (last && u == 0) {
                    // stage 0: single twiddle; fold N^-1 into both outputs
                    const double d = v[g][c] - v[g][c + half];
                    v[g][c] = mulmod(v[g][c] + v[g][c + half], C->ninv[pr], m);
                    v[g][c + half] = mulmod(d, C->itw1_ninv[pr], m);
                } else {
                    bfly_inv(v[g][c], v[g][c + half], twr[g * PER + (1 << u) - 1 + (c >> (R - u))], m);
                }
            }
        }
    }
    if constexpr (!last) {
        if constexpr (PASS == 1) load_tw<LOGN, E, 0, true>(itw, tid, twr_next);
        else load_tw<LOGN, E, PASS - 1, false>(itw, tid, twr_next);
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
        const int pb = pad(base[g]);
#pragma unroll
        for (int c = 0; c < (1 << R); c++) {
            // the last pass pairs elements N/2 apart with consecutive lanes on consecutive
            // addresses: it stores straight to global memory
            if (last) st.store(wg, base[g] + (c << L), v[g][c], m, C);
            else lds[pb + pad(c << L)] = v[g][c];
        }
    }
    if constexpr (!last) {
        if constexpr (PASS - 1 < P::NC) lds_barrier();   // the next pass reads other waves' elements
        else wave_sync();
    }
}

template <int LOGN, int E, class LD, class ST>
__global__ void __launch_bounds__((1 << LOGN) / E, (min_waves<LOGN, E>()))
ntt_inv_kernel(LD ld, ST st, const double *__restrict__ itw_all, const DevConst *__restrict__ C, int nwg)
{
    __shared__ double lds[lds_doubles<LOGN>()];
    constexpr bool PF = LD::kPrefetch && prefetch_rows<LOGN, E>();
    constexpr int NP = Plan<LOGN, E>::NP;
    static_assert(NP - 1 >= Plan<LOGN, E>::NC, "the first inverse pass must be wave-local");
    const int tid = threadIdx.x;
    const int S = ld.share(C);
    int p = blockIdx.x;
    int wg = xcd_row(p, nwg, S);
    uint64_t raw[PF ? E : 1][LD::kRaw];
    if constexpr (PF) fetch_row<LOGN, E, true>(ld, wg, tid, C, raw);
    for (;;) {
        const int pr = ld.prime(wg, C);
        const ModD m = C->mod[pr];
        const double *itw = itw_all + ((size_t)pr << LOGN);
        double twa[TWREGS], twb[TWREGS];
        load_tw<LOGN, E, NP - 1, false>(itw, tid, twa);
        {
            // each wave brings in its own chunk (consecutive lanes on consecutive addresses) and
            // re-reads it from LDS in the stride-1 pattern of the first pass
            if constexpr (PF) {
#pragma unroll
                for (int it = 0; it < E; it++) {
                    const int idx = chunk_elem<E>(tid, it);
                    lds[pad(idx)] = ld.finish(raw[it], wg, idx, m, C);
                }
            } else {
                load_row_now<LOGN, E, true>(ld, wg, tid, m, C, [&](int, int idx, double v) { lds[pad(idx)] = v; });
            }
        }
        p += (int)gridDim.x;
        const bool more = p < nwg;
        const int wg_next = more ? xcd_row(p, nwg, S) : 0;
        const int orow = ld.out_row(wg, C);
        if constexpr (PF) {
            if (more) fetch_row<LOGN, E, true>(ld, wg_next, tid, C, raw);
        }
        wave_sync();
        // passes NP-1 ... 0; the twiddle buffers alternate
        if constexpr (NP == 5) {
            inv_pass<LOGN, E, 4>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
            inv_pass<LOGN, E, 3>(lds, st, orow, tid, itw, twb, twa, m, pr, C);
            inv_pass<LOGN, E, 2>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
            inv_pass<LOGN, E, 1>(lds, st, orow, tid, itw, twb, twa, m, pr, C);
            inv_pass<LOGN, E, 0>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
        } else if constexpr (NP == 4) {
            inv_pass<LOGN, E, 3>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
            inv_pass<LOGN, E, 2>(lds, st, orow, tid, itw, twb, twa, m, pr, C);
            inv_pass<LOGN, E, 1>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
            inv_pass<LOGN, E, 0>(lds, st, orow, tid, itw, twb, twa, m, pr, C);
        } else {
            inv_pass<LOGN, E, 2>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
            inv_pass<LOGN, E, 1>(lds, st, orow, tid, itw, twb, twa, m, pr, C);
            inv_pass<LOGN, E, 0>(lds, st, orow, tid, itw, twa, twb, m, pr, C);
        }
        if (!more) break;
        wg = wg_next;
        lds_barrier();   // pass 0's LDS reads precede the next row's LDS writes
    }
}

// Inverse loaders marked here run with 16 elements per thread at N = 8192, like the forward
// transforms (two co-resident 512-thread workgroups per compute unit).  It pays for the tensor
// product, whose launches are large; the key-switch inner product is launched over a few hundred
// rows at a time and finishes a row sooner on 1024 threads.
template <class LD> struct inv_wide { static constexpr bool value = false; };

// ---------------------------------------------------------------------------
// exact base conversion helpers (per coefficient, registers only)
// ---------------------------------------------------------------------------
// x[0..ns) canonical residues -> mixed-radix digits a[0..ns); returns true when
// CENTRED and the integer exceeds floor(S/2) (its centred representative is x - S).
template <bool CENTRED>
__device__ __forceinline__ bool garner(const ConvTab &T, const DevConst *C, const double *x, double *a)
{
    a[0] = x[0];
#pragma unroll
    for (int j = 1; j < MAXS; j++) {
        if (j < T.ns) {
            const ModD mj = C->mod[T.sidx[j]];
            double v = x[j];
#pragma unroll
            for (int i = 0; i < j; i++) v = mulmod(v - a[i], T.inv[i][j], mj);
            a[j] = canon(v, mj);
        }
    }
    bool gt = false;
    if (CENTRED) {
#pragma unroll
        for (int i = 0; i < MAXS; i++)
            if (i < T.ns) gt = (a[i] > T.half[i]) || (a[i] == T.half[i] && gt);
    }
    return gt;
}
// residue of the (optionally negative-shifted) integer modulo target jt; lazy, |.| < 3p
__device__ __forceinline__ double horner(const ConvTab &T, const DevConst *C, const double *a, int jt,
                                         bool neg)
{
    const ModD mt = C->mod[T.tidx[jt]];
    double acc = 0.0;
#pragma unroll
    for (int i = MAXS - 1; i >= 0; i--) {
        if (i < T.ns) acc = (i == T.ns - 1) ? a[i] : mulmod(acc, T.s_mod_t[i][jt], mt) + a[i];
    }
    if (neg) acc -= T.S_mod_t[jt];
    return acc;
}

// compile-time-sized variants (source basis of exactly NS primes): fully unrolled, no guards
template <int NS, bool CENTRED>
__device__ __forceinline__ bool garner_t(const ConvTab &T, const DevConst *C, const double (&x)[NS], double (&a)[NS])
{
    a[0] = x[0];
#pragma unroll
    for (int j = 1; j < NS; j++) {
        const ModD mj = C->mod[T.sidx[j]];
        double v = x[j];
#pragma unroll
        for (int i = 0; i < j; i++) v = mulmod(v - a[i], T.inv[i][j], mj);
        a[j] = canon(v, mj);
    }
    bool gt = false;
    if (CENTRED) {
#pragma unroll
        for (int i = 0; i < NS; i++) gt = (a[i] > T.half[i]) || (a[i] == T.half[i] && gt);
    }
    return gt;
}
template <int NS>
__device__ __forceinline__ double horner_t(const ConvTab &T, const DevConst *C, const double (&a)[NS], int jt, bool neg)
{
    const ModD mt = C->mod[T.tidx[jt]];
    double acc = a[NS - 1];
#pragma unroll
    for (int i = NS - 2; i >= 0; i--) acc = mulmod(acc, T.s_mod_t[i][jt], mt) + a[i];
    if (neg) acc -= T.S_mod_t[jt];
    return acc;
}

// ---------------------------------------------------------------------------
// loaders / storers for the transforms
// ---------------------------------------------------------------------------
struct StF64 {      // forward output: lazy doubles
    double *base;
    __device__ __forceinline__ void store(int limb, int idx, double v, const ModD) const
    {
        base[((size_t)limb << logn) + idx] = v;
    }
    int logn;
};
struct StF64Red {   // forward output reduced to |x| <= p/2 (prepared keys and plaintexts)
    double *base;
    int logn;
    __device__ __forceinline__ void store(int limb, int idx, double v, const ModD m) const
    {
        base[((size_t)limb << logn) + idx] = red(v, m);
    }
};
struct StU64 {      // forward output: canonical uint64 (public transform entry point)
    uint64_t *base;
    int logn;
    __device__ __forceinline__ void store(int limb, int idx, double v, const ModD m) const
    {
        base[((size_t)limb << logn) + idx] = f64_to_u64(canon(v, m));
    }
};

__device__ __forceinline__ uint64_t f64_bits(double x)
{
    union { double d; uint64_t u; } v;
    v.d = x;
    return v.u;
}
__device__ __forceinline__ double bits_f64(uint64_t x)
{
    union { double d; uint64_t u; } v;
    v.u = x;
    return v.d;
}

// rows of uint64 residues, row w uses prime tab[w] (tab != null) or w % pmod
struct LdRowsU64 {
    static constexpr int kRaw = 1;
    static constexpr bool kPrefetch = true;
    static constexpr bool kScatter = false;
    const uint64_t *src;
    const uint32_t *tab;
    int pmod, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *) const { return tab ? (int)tab[wg] : wg % pmod; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int dst_limb(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *, uint64_t *raw) const
    {
        raw[0] = src[((size_t)wg << logn) + idx];
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD, const DevConst *) const
    {
        return u64_to_f64(raw[0]);
    }
};

// Inputs of a batch of tensor products.  The source ciphertexts are the n_a "a" operands followed
// by the `batch` "b" operands; polynomial pp = 2 * ciphertext + component.  Every polynomial is
// transformed once over the k ciphertext primes (LdMulQ) and the l auxiliary primes (LdMulAux) into
// ntt[pp][k+l][N]; an a operand shared by several products is transformed once.
struct MulSrc {
    const uint64_t *cta, *ctb;
    int n_a, b_group, b_stride, logn;   // b ciphertext of unit u: (u / b_group) * b_stride + u % b_group
    int dst_strided;                    // transformed rows land at the source's (strided) ciphertext index
    __device__ __forceinline__ int dst_poly(int pp) const
    {
        if (!dst_strided) return pp;
        const int u = (pp >> 1) - n_a;
        return 2 * ((u / b_group) * b_stride + u % b_group) + (pp & 1);
    }
    __device__ __forceinline__ const uint64_t *poly(int pp, int k) const
    {
        const int ct = pp >> 1, comp = pp & 1;
        const uint64_t *base;
        if (ct < n_a) base = cta + (((size_t)ct * 2 * k) << logn);
        else {
            const int u = ct - n_a;
            base = ctb + (((size_t)((u / b_group) * b_stride + u % b_group) * 2 * k) << logn);
        }
        return base + (((size_t)comp * k) << logn);
    }
};
struct LdMulQ {     // workgroup -> (pp, ciphertext prime i)
    static constexpr int kRaw = 1;
    static constexpr bool kPrefetch = true;
    static constexpr bool kScatter = false;
    MulSrc src;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return wg % C->k; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int dst_limb(int wg, const DevConst *C) const
    {
        return src.dst_poly(wg / C->k) * C->KL + wg % C->k;
    }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int k = C->k;
        raw[0] = src.poly(wg / k, k)[((size_t)(wg % k) << src.logn) + idx];
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD, const DevConst *) const
    {
        return u64_to_f64(raw[0]);
    }
};
// workgroup -> (pp, auxiliary prime j): the centred integer lift of each coefficient (exact, via
// mixed-radix digits of its K residues) reduced modulo the auxiliary prime
template <int K>
struct LdMulAux {
    static constexpr int kRaw = K;
    static constexpr bool kPrefetch = false;   // K words per element: fetched in slices instead
    static constexpr bool kScatter = false;
    MulSrc src;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return C->k + wg % C->l; }
    __device__ __forceinline__ int share(const DevConst *C) const { return C->l; }
    __device__ __forceinline__ int dst_limb(int wg, const DevConst *C) const
    {
        return src.dst_poly(wg / C->l) * C->KL + C->k + wg % C->l;
    }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const uint64_t *p = src.poly(wg / C->l, K) + idx;
#pragma unroll
        for (int i = 0; i < K; i++) raw[i] = p[(size_t)i << src.logn];
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int wg, int, const ModD mb, const DevConst *C) const
    {
        double x[K], dg[K];
#pragma unroll
        for (int i = 0; i < K; i++) x[i] = u64_to_f64(raw[i]);
        const bool neg = garner_t<K, true>(C->q2b, C, x, dg);
        return canon(horner_t<K>(C->q2b, C, dg, wg % C->l, neg), mb);
    }
};

// key-switch mod-up: workgroup -> (unit b, digit j, target prime r); the digit is
// the integer in [0,Q_j) formed by ALPHA rows of the source ring element, reduced
// modulo the target prime.  GALOIS: the source is first mapped by X -> X^galois
// (scatter through LDS; an odd multiplier permutes the LDS banks without conflicts).
// The Galois map acts on the element modulo Q: a negated coefficient is q_s - x in
// every source row, and only then is the digit lifted and reduced.
template <bool GALOIS, int ALPHA>
struct LdModup {
    static constexpr int kRaw = ALPHA;
    static constexpr bool kPrefetch = true;
    static constexpr bool kScatter = GALOIS;
    const uint64_t *src;     // ring element of unit 0
    size_t unit_stride;      // in uint64
    uint32_t galois;
    int logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return wg % C->L; }
    __device__ __forceinline__ int share(const DevConst *C) const { return C->L; }
    __device__ __forceinline__ int dst_limb(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int L = C->L, j = (wg / L) % C->dnum, b = wg / (L * C->dnum);
        const uint64_t *e = src + (size_t)b * unit_stride + idx;
#pragma unroll
        for (int s = 0; s < ALPHA; s++) raw[s] = e[(size_t)(j * ALPHA + s) << logn];
    }
    __device__ __forceinline__ int place(int idx, int n) const
    {
        const uint32_t ee = ((uint32_t)idx * galois) & (2u * n - 1);
        return (int)(ee >= (uint32_t)n ? ee - n : ee);
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int wg, int idx, const ModD mr,
                                             const DevConst *C) const
    {
        const int L = C->L, r = wg % L, j = (wg / L) % C->dnum;
        bool negate = false;
        if (GALOIS) negate = (((uint32_t)idx * galois) & ((2u << logn) - 1)) >= (1u << logn);
        double x[MAXS], a[MAXS];
#pragma unroll
        for (int s = 0; s < ALPHA; s++) {
            x[s] = u64_to_f64(raw[s]);
            if (negate) x[s] = (x[s] == 0.0) ? 0.0 : C->mod[j * ALPHA + s].p - x[s];
        }
        if (ALPHA == 1) return canon(x[0], mr);
        const ConvTab &T_ = C->dig[j];
        garner<false>(T_, C, x, a);
        return canon(horner(T_, C, a, r, false), mr);
    }
};

// plaintext polynomial mod t -> centred lift -> row modulo q_i: workgroup -> (b, i)
struct LdPlain {
    static constexpr int kRaw = 1;
    static constexpr bool kPrefetch = true;
    static constexpr bool kScatter = false;
    const uint64_t *pt;
    int logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return wg % C->k; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int dst_limb(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        raw[0] = pt[((size_t)(wg / C->k) << logn) + idx];
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD, const DevConst *C) const
    {
        const double v = u64_to_f64(raw[0]);
        return (v > 0.5 * (C->tmod - 1.0)) ? v - C->tmod : v;
    }
};

// inverse-transform loaders (finish may return any lazy value below 8p)
struct LdInvU64 {
    static constexpr int kRaw = 1;
    static constexpr bool kPrefetch = true;
    const uint64_t *src;
    const uint32_t *tab;
    int pmod, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *) const { return tab ? (int)tab[wg] : wg % pmod; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *, uint64_t *raw) const
    {
        raw[0] = src[((size_t)wg << logn) + idx];
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD, const DevConst *) const
    {
        return u64_to_f64(raw[0]);
    }
};
// key-switch inner product fused into the load: workgroup -> (unit b, prime r, component c), the
// component running fastest so that the two rows reading the same digits are neighbours;
struct LdInvTensor;
template <> struct inv_wide<LdInvTensor> { static constexpr bool value = true; };

// element = sum_j digit_j[b][r] * key[j][c][r] (both in transform order); result row [b][c][r]
template <int DNUM>
struct LdInvKsInner {
    static constexpr int kRaw = 2 * DNUM;
    static constexpr bool kPrefetch = false;
    const double *dig;   // [b][DNUM][L][N] lazy
    const double *key;   // [DNUM][2][L][N] reduced
    int logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return (wg >> 1) % C->L; }
    __device__ __forceinline__ int share(const DevConst *) const { return 2; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *C) const
    {
        const int L = C->L, r = (wg >> 1) % L, b = wg / (2 * L);
        return (b * 2 + (wg & 1)) * L + r;
    }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int L = C->L, r = (wg >> 1) % L, c = wg & 1, b = wg / (2 * L);
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            raw[2 * j] = f64_bits(dig[(((size_t)(b * DNUM + j) * L + r) << logn) + idx]);
            raw[2 * j + 1] = f64_bits(key[(((size_t)(j * 2 + c) * L + r) << logn) + idx]);
        }
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD m, const DevConst *) const
    {
        // digits are lazy (|x| <= 7.5 p), keys reduced: each product is below 1.91 p, so up to four
        // of them sum to less than 8 p without reducing the digits first
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            const double d = bits_f64(raw[2 * j]);
            s += mulmod(DNUM <= 4 ? d : red(d, m), bits_f64(raw[2 * j + 1]), m);
        }
        return s;
    }
};

// A series of rotations of the same ciphertexts ("hoisted" rotations): the digits of c1 are lifted,
// extended and transformed once, and every Galois element is applied to the transformed digits,
// where it is a permutation of the evaluation points: row element i is the value at
// psi^(2 bitrev(i) + 1), and sigma_g(a) takes there the value of a at psi^((2 bitrev(i) + 1) g).
constexpr int MAXROT = 128;   // rotations per launch
struct HoistTab {
    uint32_t g[MAXROT];            // Galois element of rotation i (inner product), its inverse mod 2N (mod-down)
    const double *key[MAXROT];     // prepared key of rotation i
};
// inner product of rotation i of unit b: workgroup -> (unit u = i * batch + b, prime r, component c);
// element = sum_j digit_j[b][r][pi_g(idx)] * key_i[j][c][r][idx]; result row [u][c][r]
template <int DNUM>
struct LdInvKsInnerHoisted {
    static constexpr int kRaw = 2 * DNUM;
    static constexpr bool kPrefetch = false;
    const double *dig;   // [b][DNUM][L][N] lazy, transform order
    HoistTab T;
    int batch, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return (wg >> 1) % C->L; }
    __device__ __forceinline__ int share(const DevConst *) const { return 2; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *C) const
    {
        const int L = C->L, r = (wg >> 1) % L, u = wg / (2 * L);
        return (u * 2 + (wg & 1)) * L + r;
    }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int L = C->L, r = (wg >> 1) % L, c = wg & 1, u = wg / (2 * L);
        const int i = u / batch, b = u - i * batch;
        const uint32_t e = ((2u * (__brev((uint32_t)idx) >> (32 - logn)) + 1u) * T.g[i]) & ((2u << logn) - 1u);
        const int sidx = (int)(__brev(e >> 1) >> (32 - logn));
        const double *kb = T.key[i];
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            raw[2 * j] = f64_bits(dig[(((size_t)(b * DNUM + j) * L + r) << logn) + sidx]);
            raw[2 * j + 1] = f64_bits(kb[(((size_t)(j * 2 + c) * L + r) << logn) + idx]);
        }
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD m, const DevConst *) const
    {
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            const double d = bits_f64(raw[2 * j]);
            s += mulmod(DNUM <= 4 ? d : red(d, m), bits_f64(raw[2 * j + 1]), m);
        }
        return s;
    }
};

// The sum of a series of rotations of one ciphertext, as one key-switch accumulator: workgroup ->
// (unit b, prime r, component c); element = sum_i sum_j digit_j[b][r][pi_{g_i}(idx)] * key_i[j][c][r][idx];
// result row [b][c][r].  Summing before the inverse transform and the division by P costs one
// inverse transform and one mod-down per ciphertext instead of one per rotation.
template <int DNUM>
struct LdInvKsInnerSum {
    static constexpr int kRaw = 2 * DNUM;
    static constexpr bool kPrefetch = false;
    const double *dig;   // [b][DNUM][L][N] lazy, transform order
    HoistTab T;
    int n_rot, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return (wg >> 1) % C->L; }
    __device__ __forceinline__ int share(const DevConst *) const { return 2; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *C) const
    {
        const int L = C->L, r = (wg >> 1) % L, b = wg / (2 * L);
        return (b * 2 + (wg & 1)) * L + r;
    }
    __device__ __forceinline__ int rounds() const { return n_rot; }
    __device__ __forceinline__ void fetch_round(int wg, int idx, int i, const DevConst *C, uint64_t *raw) const
    {
        const int L = C->L, r = (wg >> 1) % L, c = wg & 1, b = wg / (2 * L);
        const uint32_t e = ((2u * (__brev((uint32_t)idx) >> (32 - logn)) + 1u) * T.g[i]) & ((2u << logn) - 1u);
        const int sidx = (int)(__brev(e >> 1) >> (32 - logn));
        const double *kb = T.key[i];
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            raw[2 * j] = f64_bits(dig[(((size_t)(b * DNUM + j) * L + r) << logn) + sidx]);
            raw[2 * j + 1] = f64_bits(kb[(((size_t)(j * 2 + c) * L + r) << logn) + idx]);
        }
    }
    __device__ __forceinline__ void fetch(int, int, const DevConst *, uint64_t *) const {}
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD m, const DevConst *) const
    {
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < DNUM; j++) {
            const double d = bits_f64(raw[2 * j]);
            s += mulmod(DNUM <= 4 ? d : red(d, m), bits_f64(raw[2 * j + 1]), m);
        }
        return s;
    }
    // one rotation's products are below 1.91 DNUM p; with the running sum reduced to p/2 first the
    // total stays below 8 p for DNUM <= 3, and for more digits the new term is reduced as well
    __device__ __forceinline__ double join(double sum, double term, const ModD m) const
    {
        return red(sum, m) + (DNUM <= 3 ? term : red(term, m));
    }
};
template <int DNUM> struct ld_rounds<LdInvKsInnerSum<DNUM>> { static constexpr bool value = true; };

// tensor product fused into the load: workgroup -> (unit u, prime r of the k+l, component c in 0..2),
// the component running fastest so that the three rows reading the same four operand rows are
// neighbours; element = a0 b0 (c = 0), a0 b1 + a1 b0 (c = 1), a1 b1 (c = 2); result row [u][c][r].
// a polys of unit u: ntt[2 * (u / a_group) + {0,1}]; b polys: ntt[2 * (n_a + u) + {0,1}], or, with
// bext given, the transformed ciphertext bext[(u / b_group) * b_stride + u % b_group].
struct LdInvTensor {
    static constexpr int kRaw = 4;
    static constexpr bool kPrefetch = false;
    const double *ntt, *bext;
    int a_group, n_a, b_group, b_stride, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return (wg / 3) % C->KL; }
    __device__ __forceinline__ int share(const DevConst *) const { return 3; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *C) const
    {
        const int KL = C->KL, r = (wg / 3) % KL, u = wg / (3 * KL);
        return (u * 3 + wg % 3) * KL + r;
    }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int KL = C->KL, c = wg % 3, r = (wg / 3) % KL, u = wg / (3 * KL);
        const size_t ps = (size_t)KL << logn, off = ((size_t)r << logn) + idx;
        const double *sa = ntt + (size_t)(2 * (u / a_group)) * ps + off;
        const double *sb = (bext ? bext + (size_t)(2 * ((u / b_group) * b_stride + u % b_group)) * ps
                                 : ntt + (size_t)(2 * (n_a + u)) * ps) + off;
        // c = 0: a0 b0; c = 2: a1 b1; c = 1: all four
        raw[0] = f64_bits(sa[c == 2 ? ps : 0]);
        raw[1] = f64_bits(sb[c == 2 ? ps : (c == 1 ? ps : 0)]);
        if (c == 1) {
            raw[2] = f64_bits(sa[ps]);
            raw[3] = f64_bits(sb[0]);
        }
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int wg, int, const ModD m, const DevConst *) const
    {
        // forward outputs are lazy: bring them to p/2 so that the two-term sum stays far below 2^53
        double s = mulmod(red(bits_f64(raw[0]), m), red(bits_f64(raw[1]), m), m);
        if (wg % 3 == 1) s += mulmod(red(bits_f64(raw[2]), m), red(bits_f64(raw[3]), m), m);
        return s;
    }
};

// The tensor products of a group of consecutive units summed before the inverse transform (and so
// before the one scaling that follows): workgroup -> (group g, prime r, component c); element =
// sum over the group's units u = g * group + i of the element LdInvTensor forms for u; result row
// [g][c][r].  Operand addressing as in LdInvTensor.
struct LdInvTensorSum {
    static constexpr int kRaw = 4;
    static constexpr bool kPrefetch = false;
    LdInvTensor one;
    int group;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return (wg / 3) % C->KL; }
    __device__ __forceinline__ int share(const DevConst *) const { return 3; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *C) const { return one.out_row(wg, C); }
    __device__ __forceinline__ int rounds() const { return group; }
    __device__ __forceinline__ void fetch_round(int wg, int idx, int i, const DevConst *C, uint64_t *raw) const
    {
        const int per = 3 * C->KL, g = wg / per;
        one.fetch((g * group + i) * per + wg % per, idx, C, raw);
    }
    __device__ __forceinline__ void fetch(int, int, const DevConst *, uint64_t *) const {}
    __device__ __forceinline__ double finish(const uint64_t *raw, int wg, int idx, const ModD m, const DevConst *C) const
    {
        return one.finish(raw, wg, idx, m, C);     // only wg % 3 matters there
    }
    // a unit's term is below 1.2 p (two products of operands reduced to p/2)
    __device__ __forceinline__ double join(double sum, double term, const ModD m) const { return red(sum, m) + term; }
};
template <> struct ld_rounds<LdInvTensorSum> { static constexpr bool value = true; };

// transformed ciphertext row times prepared plaintext row (ct x pt fused into the load):
// workgroup -> (unit b, comp c, prime i); ciphertext = ctf[b / ct_group], plaintext =
// plain[(b % p_mod) * pstride + pofs]
struct LdInvMulPlain {
    static constexpr int kRaw = 2;
    static constexpr bool kPrefetch = true;
    const double *ctf;     // forward-transformed ciphertext rows [*][2][k][N]
    const double *plain;   // prepared plaintexts [*][k][N]
    int ct_group, p_mod, pstride, pofs, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return wg % C->k; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int wg, int idx, const DevConst *C, uint64_t *raw) const
    {
        const int k = C->k, i = wg % k, c = (wg / k) & 1, b = wg / (2 * k);
        raw[0] = f64_bits(ctf[((size_t)(((b / ct_group) * 2 + c) * k + i) << logn) + idx]);
        raw[1] = f64_bits(plain[((size_t)(((b % p_mod) * pstride + pofs) * k + i) << logn) + idx]);
    }
    __device__ __forceinline__ double finish(const uint64_t *raw, int, int, const ModD m, const DevConst *) const
    {
        return mulmod(bits_f64(raw[0]), bits_f64(raw[1]), m);
    }
};

// sum of ciphertext-plaintext products fused into the load (the decode step's vector-matrix
// product): workgroup -> (unit u, comp c2, prime i); element = sum over the cn rotated copies of
// the token of copy_c[c2][i] * diagonal_(u, c)[i].  The 2 cn operands of an element are read
// where they are used (they would not fit the register slices of the other loaders); the copies
// are stored reduced, so every product is below 0.6 p and eight of them sum to less than 5 p.
struct LdInvPlainSum {
    static constexpr int kRaw = 1;
    static constexpr bool kPrefetch = false;
    const double *ctf;     // transformed copies [cn][2][k][N], |x| <= p/2
    const double *plain;   // prepared plaintexts [units][cn][k][N]
    int cn, logn;
    __device__ __forceinline__ int prime(int wg, const DevConst *C) const { return wg % C->k; }
    __device__ __forceinline__ int share(const DevConst *) const { return 1; }
    __device__ __forceinline__ int out_row(int wg, const DevConst *) const { return wg; }
    __device__ __forceinline__ void fetch(int, int, const DevConst *, uint64_t *raw) const { raw[0] = 0; }
    __device__ __forceinline__ double finish(const uint64_t *, int wg, int idx, const ModD m, const DevConst *C) const
    {
        const int k = C->k, i = wg % k, c2 = (wg / k) & 1, u = wg / (2 * k);
        const double *a = ctf + ((size_t)(c2 * k + i) << logn) + idx;
        const double *b = plain + ((((size_t)u * cn) * k + i) << logn) + idx;
        const size_t sa = (size_t)(2 * k) << logn, sb = (size_t)k << logn;
        double s = 0.0;
        for (int c = 0; c < cn; c++) {
            s += mulmod(a[c * sa], b[c * sb], m);
            if ((c & 7) == 7) s = red(s, m);
        }
        return s;
    }
};

struct StInvF64 {
    double *dst;
    int logn;
    __device__ __forceinline__ void store(int wg, int idx, double v, const ModD, const DevConst *) const
    {
        dst[((size_t)wg << logn) + idx] = v;
    }
};
struct StInvU64 {
    uint64_t *dst;
    int logn;
    __device__ __forceinline__ void store(int wg, int idx, double v, const ModD m, const DevConst *) const
    {
        dst[((size_t)wg << logn) + idx] = f64_to_u64(canon(v, m));
    }
};
// cache append: workgroup -> (cache c, comp, prime); target row = cache + c*stride + row;
// fresh != 0 stores, otherwise adds to what is there
struct StInvAppend {
    uint64_t *cache;        // first target ciphertext (cache 0)
    size_t cache_stride;    // uint64 between consecutive caches' target ciphertexts
    int fresh, logn;
    __device__ __forceinline__ void store(int wg, int idx, double v, const ModD m, const DevConst *C) const
    {
        const int rows = 2 * C->k, c = wg / rows, row = wg % rows;
        uint64_t *p = cache + (size_t)c * cache_stride + ((size_t)row << logn) + idx;
        double r = canon(v, m);
        if (!fresh) r = addmod_canon(r, u64_to_f64(*p), m);
        *p = f64_to_u64(r);
    }
};

// ---------------------------------------------------------------------------
// pointwise kernels
// ---------------------------------------------------------------------------
constexpr int PW_THREADS = 256;

// exact round(t e / Q) mod Q from e known modulo Q and the auxiliary basis:
//   r = centred (t e mod Q);  y = (t e - r) / Q computed modulo each b_j;
//   y is below B/2 in magnitude, so its centred lift from the auxiliary basis is exact.
// tens[b*3+c][r][n] (lazy, coefficient order) -> out[b][c][i][n] canonical uint64;
// acc != 0 adds the result to what out already holds (sum of products).
template <int K>
__global__ void __launch_bounds__(PW_THREADS)
scale_kernel(const double *__restrict__ tens, uint64_t *__restrict__ out, int total_polys, int acc,
             const DevConst *__restrict__ C)
{
    constexpr int L = K + 1;
    const int logn = C->logn, N = 1 << logn;
    const size_t gid = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    const int n = (int)(gid & (N - 1));
    const int bc = (int)(gid >> logn);
    if (bc >= total_polys) return;
    const double *src = tens + (((size_t)bc * (K + L)) << logn) + n;
    const double t = C->tmod;
    double e[K + L];
#pragma unroll
    for (int i = 0; i < K + L; i++) e[i] = src[(size_t)i << logn];
    double x[K], dq[K], y[L], db[L];
#pragma unroll
    for (int i = 0; i < K; i++) x[i] = canon(mulmod(e[i], t, C->mod[i]), C->mod[i]);
    const bool neg = garner_t<K, true>(C->q2b, C, x, dq);
#pragma unroll
    for (int j = 0; j < L; j++) {
        const ModD mb = C->mod[K + j];
        const double te = mulmod(e[K + j], t, mb);
        const double rj = horner_t<K>(C->q2b, C, dq, j, neg);
        y[j] = canon(mulmod(red(te - rj, mb), C->Qinv_b[j], mb), mb);
    }
    const bool neg2 = garner_t<L, true>(C->b2q, C, y, db);
    uint64_t *o = out + (((size_t)bc * K) << logn) + n;
#pragma unroll
    for (int i = 0; i < K; i++) {
        double v = canon(horner_t<L>(C->b2q, C, db, i, neg2), C->mod[i]);
        if (acc) v = addmod_canon(v, u64_to_f64(o[(size_t)i << logn]), C->mod[i]);
        o[(size_t)i << logn] = f64_to_u64(v);
    }
}

// mod-down with rounding and the final additions of relinearisation / rotation:
//   u = floor((A + floor(P/2)) / P) mod Q,  out[b][c] = u (+ add0) (+ add1)
// add0: relin -> in3[b][c];  rotate -> sigma_g(in2[b][0]) for c = 0, nothing for c = 1
// add1: rotate with accumulate -> acc_add[b][c] (the rotated ciphertext itself, or another one)
struct ModdownArgs {
    const double *acc;        // [b][2][L][N] lazy, coefficient order
    uint64_t *out;            // unit b at out + b*out_stride, [2][k][N]
    size_t out_stride;
    const uint64_t *add;      // base of the addend ciphertexts (unit 0) or null
    size_t add_stride;        // uint64 per unit in add
    uint32_t galois;          // != 0: add is permuted by X -> X^galois and only applies to c = 0
    int accumulate;           // also add the un-permuted acc_add[b][c]
    int batch;
    const uint64_t *acc_add;  // base of the ciphertexts added un-permuted (accumulate)
    size_t acc_stride;
};
// HOIST: the units are the rotations of a series, unit u = i * rot_batch + b being rotation i of
// ciphertext b: its Galois element comes from the table, its addend is ciphertext b and its output
// ciphertext b * out_per_b + i.
// n_sum: rotations whose accumulators were summed (moddown_sum_kernel).
template <int LOGN> constexpr int moddown_sum_split() { return (1 << LOGN) / 2048 >= 4 ? 4 : (1 << LOGN) / 2048; }
struct ModdownHoist {
    uint32_t ginv[MAXROT];
    int rot_batch, out_per_b, n_sum;
};
template <bool HOIST>
__global__ void __launch_bounds__(PW_THREADS)
moddown_kernel(ModdownArgs A, ModdownHoist H, const DevConst *__restrict__ C)
{
    // a thread takes two neighbouring coefficients: 16 bytes per row and lane on every read and
    // write that is not a permuted one
    const int logn = C->logn, N = 1 << logn, k = C->k, nsp = C->nsp, L = C->L;
    // the N / (2 PW_THREADS) blocks of one (unit, component) run on one XCD: the permuted reads of a
    // c0 row touch all of its cache lines, which that XCD's L2 then fetches once instead of once
    // per XCD
    const size_t gid =
        ((size_t)xcd_row((int)blockIdx.x, (int)gridDim.x, N / (2 * PW_THREADS)) * PW_THREADS + threadIdx.x) * 2;
    const int n = (int)(gid & (N - 1));
    const int bc = (int)(gid >> logn);
    if (bc >= A.batch * 2) return;
    const int c = bc & 1;
    int b = bc >> 1, bo = b;       // addend index, output index
    if (HOIST) {
        const int i = b / H.rot_batch;
        b -= i * H.rot_batch;
        bo = b * H.out_per_b + i;
        A.galois = H.ginv[i];
    }
    const double *src = A.acc + (((size_t)bc * L) << logn) + n;
    double xp[2][MAXS], dg[2][MAXS];
#pragma unroll
    for (int s = 0; s < 2; s++)
        if (s < nsp) {
            const ModD mp = C->mod[k + s];
            const double2 x2 = *reinterpret_cast<const double2 *>(src + ((size_t)(k + s) << logn));
            xp[0][s] = addmod_canon(canon(x2.x, mp), C->halfP[k + s], mp);
            xp[1][s] = addmod_canon(canon(x2.y, mp), C->halfP[k + s], mp);
        }
    garner<false>(C->p2q, C, xp[0], dg[0]);
    garner<false>(C->p2q, C, xp[1], dg[1]);
    int src_idx[2] = {0, 0};
    bool negate[2] = {false, false};
    if (A.galois) {
        // inverse map: output index n takes the coefficient from index n * g^-1 mod 2N
        // (A.galois already holds g^-1 mod 2N)
#pragma unroll
        for (int e2 = 0; e2 < 2; e2++) {
            const uint32_t e = ((uint32_t)(n + e2) * A.galois) & (2 * N - 1);
            negate[e2] = e >= (uint32_t)N;
            src_idx[e2] = (int)(negate[e2] ? e - N : e);
        }
    }
    uint64_t *o = A.out + (size_t)bo * A.out_stride + (((size_t)c * k) << logn) + n;
#pragma unroll
    for (int i = 0; i < MAXS; i++)
        if (i < k) {
            const ModD mq = C->mod[i];
            const double2 a2 = *reinterpret_cast<const double2 *>(src + ((size_t)i << logn));
            const double ain[2] = {a2.x, a2.y};
            double v[2];
#pragma unroll
            for (int e2 = 0; e2 < 2; e2++) {
                const double ai = addmod_canon(canon(ain[e2], mq), C->halfP[i], mq);
                const double ri = horner(C->p2q, C, dg[e2], i, false);
                v[e2] = canon(mulmod(red(ai - ri, mq), C->Pinv_q[i], mq), mq);
            }
            if (A.add) {
                const uint64_t *ad = A.add + (size_t)b * A.add_stride;
                if (A.galois) {
                    if (c == 0) {
#pragma unroll
                        for (int e2 = 0; e2 < 2; e2++) {
                            double w = u64_to_f64(ad[((size_t)i << logn) + src_idx[e2]]);
                            if (negate[e2]) w = (w == 0.0) ? 0.0 : mq.p - w;
                            v[e2] = addmod_canon(v[e2], w, mq);
                        }
                    }
                    if (A.accumulate) {
                        const uint64_t *aa = A.acc_add + (size_t)b * A.acc_stride;
                        const ulonglong2 w2 =
                            *reinterpret_cast<const ulonglong2 *>(aa + ((size_t)(c * k + i) << logn) + n);
                        v[0] = addmod_canon(v[0], u64_to_f64(w2.x), mq);
                        v[1] = addmod_canon(v[1], u64_to_f64(w2.y), mq);
                    }
                } else {
                    const ulonglong2 w2 = *reinterpret_cast<const ulonglong2 *>(ad + ((size_t)(c * k + i) << logn) + n);
                    v[0] = addmod_canon(v[0], u64_to_f64(w2.x), mq);
                    v[1] = addmod_canon(v[1], u64_to_f64(w2.y), mq);
                }
            }
            *reinterpret_cast<ulonglong2 *>(o + ((size_t)i << logn)) = make_ulonglong2(f64_to_u64(v[0]), f64_to_u64(v[1]));
        }
}

// Mod-down of a summed series of rotations (acc holds the summed accumulators of the H.n_sum
// rotations of ciphertext b), one output row per workgroup: block -> (ciphertext b, component c,
// ciphertext prime i), the prime running fastest.
//   out[b][c][i] = in[b][c][i] + u_{c,i} + [c = 0] sum_r sigma_r(c0)_i
// The Galois maps read c0 at the indices n g_r^-1 mod 2N, a different cache line for every lane;
// the workgroup brings its input row into LDS with coalesced loads and takes the permuted
// coefficients (and the un-permuted addend) from there.  Base conversion as in moddown_kernel,
// for the one prime of the row; the special-prime rows are read by the k workgroups of a
// (ciphertext, component), neighbours on one XCD.
template <int LOGN>
__global__ void __launch_bounds__(1024, (LOGN <= 13 ? 8 : 4))
moddown_sum_kernel(ModdownArgs A, ModdownHoist H, const DevConst *__restrict__ C)
{
    // a row is shared by SPLIT workgroups: each parks the whole input row in LDS and produces
    // N / SPLIT of the outputs (SPLIT x k workgroups per ciphertext and component)
    constexpr int N = 1 << LOGN, SPLIT = moddown_sum_split<LOGN>(), ROWP = N / 2048, PAIRS = ROWP / SPLIT;
    static_assert(PAIRS >= 1, "at least one pair of outputs per thread");
    __shared__ double row[N];
    const int k = C->k, nsp = C->nsp, L = C->L, tid = threadIdx.x;
    const int blk = xcd_row((int)blockIdx.x, (int)gridDim.x, k * SPLIT);
    const int part = blk % SPLIT, i = (blk / SPLIT) % k, bc = blk / (SPLIT * k), c = bc & 1, b = bc >> 1;
    const ModD mq = C->mod[i];
    const uint64_t *in = A.add + (size_t)b * A.add_stride + ((size_t)(c * k + i) << LOGN);   // row i of c_c
    const double *acc = A.acc + (((size_t)bc * L) << LOGN);
    uint64_t *o = A.out + (size_t)b * A.out_stride + ((size_t)(c * k + i) << LOGN);
    // the input row (component 1: only the part this workgroup produces), and the accumulator
    // operands of the thread's first pairs, are requested before anything waits
    auto pair_index = [&](int j) { return 2 * (tid + 1024 * (part * PAIRS + j)); };
    if (c == 0) {
        ulonglong2 all[ROWP];
#pragma unroll
        for (int j = 0; j < ROWP; j++) all[j] = *reinterpret_cast<const ulonglong2 *>(in + 2 * (tid + 1024 * j));
#pragma unroll
        for (int j = 0; j < ROWP; j++)
            *reinterpret_cast<double2 *>(row + 2 * (tid + 1024 * j)) =
                make_double2(u64_to_f64(all[j].x), u64_to_f64(all[j].y));
    } else {
#pragma unroll
        for (int j = 0; j < PAIRS; j++) {
            const ulonglong2 w = *reinterpret_cast<const ulonglong2 *>(in + pair_index(j));
            *reinterpret_cast<double2 *>(row + pair_index(j)) = make_double2(u64_to_f64(w.x), u64_to_f64(w.y));
        }
    }
    constexpr int PB = PAIRS < 2 ? PAIRS : 2;
    double2 xs[PB][2], as[PB];
    auto request = [&](int j0) {
#pragma unroll
        for (int j = 0; j < PB; j++) {
            const int n = pair_index(j0 + j);
#pragma unroll
            for (int s = 0; s < 2; s++)
                if (s < nsp) xs[j][s] = *reinterpret_cast<const double2 *>(acc + ((size_t)(k + s) << LOGN) + n);
            as[j] = *reinterpret_cast<const double2 *>(acc + ((size_t)i << LOGN) + n);
        }
    };
    request(0);
    if (c == 0) __syncthreads();     // component 1 reads back only its own elements
#pragma unroll
    for (int j0 = 0; j0 < PAIRS; j0 += PB) {
        double v[PB][2];
#pragma unroll
        for (int j = 0; j < PB; j++) {
            double xp[2][MAXS], dg[2][MAXS];
#pragma unroll
            for (int s = 0; s < 2; s++)
                if (s < nsp) {
                    const ModD mp = C->mod[k + s];
                    xp[0][s] = addmod_canon(canon(xs[j][s].x, mp), C->halfP[k + s], mp);
                    xp[1][s] = addmod_canon(canon(xs[j][s].y, mp), C->halfP[k + s], mp);
                }
            garner<false>(C->p2q, C, xp[0], dg[0]);
            garner<false>(C->p2q, C, xp[1], dg[1]);
            const double ain[2] = {as[j].x, as[j].y};
#pragma unroll
            for (int e2 = 0; e2 < 2; e2++) {
                const double ai = addmod_canon(canon(ain[e2], mq), C->halfP[i], mq);
                const double ri = horner(C->p2q, C, dg[e2], i, false);
                v[j][e2] = canon(mulmod(red(ai - ri, mq), C->Pinv_q[i], mq), mq);
            }
        }
        if (j0 + PB < PAIRS) request(j0 + PB);     // the next pairs' operands travel during the LDS reads
#pragma unroll
        for (int j = 0; j < PB; j++) {
            const int n = pair_index(j0 + j);
            if (c == 0)
                for (int r = 0; r < H.n_sum; r++) {
                    const uint32_t gi = H.ginv[r];
#pragma unroll
                    for (int e2 = 0; e2 < 2; e2++) {
                        const uint32_t e = ((uint32_t)(n + e2) * gi) & (2 * N - 1);
                        const bool ng = e >= (uint32_t)N;
                        double w = row[ng ? e - N : e];
                        if (ng) w = (w == 0.0) ? 0.0 : mq.p - w;
                        v[j][e2] = addmod_canon(v[j][e2], w, mq);
                    }
                }
            const double2 own = *reinterpret_cast<const double2 *>(row + n);
            v[j][0] = addmod_canon(v[j][0], own.x, mq);
            v[j][1] = addmod_canon(v[j][1], own.y, mq);
            *reinterpret_cast<ulonglong2 *>(o + n) = make_ulonglong2(f64_to_u64(v[j][0]), f64_to_u64(v[j][1]));
        }
    }
}

// out = a + b over `rows` rows of N residues, row w modulo q_(w % k)
__global__ void __launch_bounds__(PW_THREADS)
add_kernel(const uint64_t *__restrict__ a, const uint64_t *__restrict__ b, uint64_t *__restrict__ out,
           int rows, const DevConst *__restrict__ C)
{
    const int logn = C->logn, N = 1 << logn;
    const size_t gid = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    const int row = (int)(gid >> logn);
    if (row >= rows) return;
    (void)N;
    const ModD m = C->mod[row % C->k];
    out[gid] = f64_to_u64(addmod_canon(u64_to_f64(a[gid]), u64_to_f64(b[gid]), m));
}

// out[b] = in[b] + sign * floor(Q/t) * pt  (the plaintext enters component 0 only; component 1 is
// copied): rows = batch * 2 * k, pt[(b % p_mod)][N] coefficients in [0, t)
__global__ void __launch_bounds__(PW_THREADS)
add_plain_kernel(const uint64_t *__restrict__ in, const uint64_t *__restrict__ pt, uint64_t *__restrict__ out,
                 int batch, int p_mod, int negative, const DevConst *__restrict__ C)
{
    const int logn = C->logn, N = 1 << logn, k = C->k;
    const size_t gid = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    const int n = (int)(gid & (N - 1));
    const int row = (int)(gid >> logn);
    if (row >= batch * 2 * k) return;
    const int i = row % k, c = (row / k) & 1, b = row / (2 * k);
    double v = u64_to_f64(in[gid]);
    if (c == 0) {
        const ModD m = C->mod[i];
        const double d = canon(mulmod(u64_to_f64(pt[((size_t)(b % p_mod) << logn) + n]), C->delta_q[i], m), m);
        v = negative ? (v >= d ? v - d : v - d + m.p) : addmod_canon(v, d, m);
    }
    out[gid] = f64_to_u64(v);
}

// out[g][e] = sum_{c < group} in[g*group + c][e] over rows*N elements per unit (row w mod q_(w%k))
__global__ void __launch_bounds__(PW_THREADS)
sum_groups_kernel(const uint64_t *__restrict__ in, uint64_t *__restrict__ out, int groups, int group,
                  int rows, const DevConst *__restrict__ C)
{
    const int logn = C->logn;
    const size_t per = (size_t)rows << logn;
    const size_t gid = (size_t)blockIdx.x * PW_THREADS + threadIdx.x;
    if (gid >= per * (size_t)groups) return;
    const size_t g = gid / per, e = gid % per;
    const ModD m = C->mod[(int)(e >> logn) % C->k];
    double s = u64_to_f64(in[(g * group) * per + e]);
    for (int c = 1; c < group; c++) s = addmod_canon(s, u64_to_f64(in[(g * group + c) * per + e]), m);
    out[gid] = f64_to_u64(s);
}

// Exchange micro-benchmark: the wave-local regrouping a transform pass boundary needs when the
// next stage pairs elements 32 lanes apart.  Every lane holds 16 doubles; one exchange hands the
// upper 8 of lanes 0-31 to lanes 32-63 in return for their lower 8 (afterwards a lane holds both
// halves of 8 butterflies).  kind 0: through the wave's own region of LDS (8 stores, wave-level
// ordering, 8 loads per lane); kind 1: v_permlane32_swap on the 32-bit halves (16 instructions per
// lane, no memory).  One add per held double between exchanges keeps the values moving.
typedef unsigned cg_uint2v __attribute__((ext_vector_type(2)));
__global__ void __launch_bounds__(1024)
bench_exchange_kernel(int kind, uint32_t iters, double *__restrict__ out)
{
    __shared__ double lds[16 * 64 * 8];
    const int tid = threadIdx.x, lane = tid & 63;
    double *mine = lds + (tid >> 6) * (64 * 8);
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; k++) v[k] = (double)(tid * 16 + k);
    for (uint32_t i = 0; i < iters; i++) {
        if (kind == 0) {
            // a lane gives away its upper half (lanes 0-31) or its lower half (lanes 32-63)
#pragma unroll
            for (int k = 0; k < 8; k++) mine[k * 64 + lane] = lane < 32 ? v[8 + k] : v[k];
            wave_sync();
#pragma unroll
            for (int k = 0; k < 8; k++) {
                const double got = mine[k * 64 + (lane ^ 32)];
                if (lane < 32) v[8 + k] = got;
                else v[k] = got;
            }
            wave_sync();
        } else {
#pragma unroll
            for (int k = 0; k < 8; k++) {
                uint64_t a = f64_bits(v[k]), b = f64_bits(v[8 + k]);
                // upper 32 lanes of the first operand <-> lower 32 lanes of the second
                const cg_uint2v lo = __builtin_amdgcn_permlane32_swap((unsigned)a, (unsigned)b, false, false);
                const cg_uint2v hi = __builtin_amdgcn_permlane32_swap((unsigned)(a >> 32), (unsigned)(b >> 32), false, false);
                v[k] = bits_f64(((uint64_t)hi.x << 32) | lo.x);
                v[8 + k] = bits_f64(((uint64_t)hi.y << 32) | lo.y);
            }
        }
#pragma unroll
        for (int k = 0; k < 16; k++) v[k] += 1.0;
    }
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < 16; k++) s += v[k] * (double)(k + 1);
    out[(size_t)blockIdx.x * blockDim.x + tid] = s;
}

// arithmetic micro-benchmark: `iters` dependent products per lane
__global__ void __launch_bounds__(PW_THREADS)
bench_modmul_kernel(int kind, uint32_t n_lanes, uint32_t iters, uint64_t *__restrict__ out, ModD md, ModI mi)
{
    const uint32_t gid = blockIdx.x * PW_THREADS + threadIdx.x;
    if (gid >= n_lanes) return;
    const uint64_t x0 = (0x9E3779B97F4A7C15ull * (gid + 1)) % mi.q;
    const uint64_t w0 = (0xD1B54A32D192ED03ull * (gid + 7)) % mi.q;
    if (kind == 0) {
        double x = u64_to_f64(x0), y = u64_to_f64(w0);
        const double w = u64_to_f64(w0);
        for (uint32_t i = 0; i < iters; i++) {
            x = mulmod(x, w, md);
            y = mulmod(y, x, md);
        }
        out[gid] = f64_to_u64(canon(x, md)) ^ f64_to_u64(canon(y, md));
    } else {
        uint64_t x = x0, y = w0;
        for (uint32_t i = 0; i < iters; i++) {
            x = mulmod_barrett(x, w0, mi);
            y = mulmod_barrett(y, x, mi);
        }
        out[gid] = x ^ y;
    }
}

}  // namespace cg
