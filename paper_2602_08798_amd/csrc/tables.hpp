// Constant tables shared by host set-up code and device kernels (layout only;
// the host fills them in cryptogen.hip, kernels read them through a pointer
// to one DevConst object in device memory).
#pragma once
#include "modarith.hpp"

namespace cg {

constexpr int MAXS = 7;    // largest source basis of an exact base conversion (l <= 7)
constexpr int MAXT = 8;    // largest target basis (k + nsp <= 8)
constexpr int MAXPR = 16;  // ciphertext + special + auxiliary primes
constexpr int MAXDIG = 6;

// Exact conversion of an integer known by its residues modulo the source basis
// S = {s_0..s_{ns-1}} into residues modulo each target prime, through
// mixed-radix (Garner) digits:  x = a_0 + s_0 (a_1 + s_1 (a_2 + ...)), 0 <= a_i < s_i.
// The digits order integers lexicographically, so comparing them with the
// digits of floor(S/2) decides the sign of the centred representative exactly.
struct ConvTab {
    int ns, nt;
    int sidx[MAXS];              // prime index of s_i
    int tidx[MAXT];              // prime index of target j
    double inv[MAXS][MAXS];      // inv[i][j] = s_i^-1 mod s_j for i < j (centred)
    double half[MAXS];           // mixed-radix digits of floor(S/2)
    double s_mod_t[MAXS][MAXT];  // s_i mod t_j (centred)
    double S_mod_t[MAXT];        // S mod t_j (centred)
};

struct DevConst {
    int logn, k, nsp, l, alpha, dnum;
    int L;    // k + nsp   (key-switching basis)
    int KL;   // k + l     (tensor basis: ciphertext primes + auxiliary primes)
    int np;   // distinct primes in mod[]: q_0..q_{k-1}, then the auxiliary basis
              // (special primes first, then private extra primes)
    ModD mod[MAXPR];
    double ninv[MAXPR];       // N^-1 mod prime (centred)
    double itw1_ninv[MAXPR];  // (first inverse twiddle) * N^-1 (centred)
    double tmod;              // plaintext modulus t
    ConvTab q2b;              // Q -> auxiliary basis, centred
    ConvTab b2q;              // auxiliary basis -> Q, centred
    double Qinv_b[MAXS];      // Q^-1 mod b_j (centred)
    ConvTab dig[MAXDIG];      // digit j (alpha primes) -> all k+nsp primes, non-centred
    ConvTab p2q;              // special primes -> Q, non-centred
    double halfP[MAXT];       // floor(P/2) mod each of the k+nsp primes (canonical)
    double Pinv_q[MAXS];      // P^-1 mod q_i (centred)
    double delta_q[MAXS];     // floor(Q/t) mod q_i (centred): the scale of a plaintext inside a ciphertext
};

}  // namespace cg
