// Constants of Section 4.1 and the shift table of Section 4.2, per number of
// moduli.  Host side only; the kernels receive copies through their arguments.
#pragma once
#include <cstdint>

namespace oz2 {

constexpr int kMinModuli = 2;
constexpr int kMaxModuli = 20;
constexpr int kMaxLevels = 20;

struct Table {
    int32_t n;                          // number of moduli
    int32_t p[kMaxModuli];              // moduli, descending from 256
    uint32_t pinv_prime[kMaxModuli];    // floor(2^32/p - 1)            (Section 4.3)
    double pinv[kMaxModuli];            // double(1/p)                  (Section 4.2)
    double s1[kMaxModuli], s2[kMaxModuli];  // split of (P/p_i) q_i     (Eq. 6)
    double P1, P2, Pinv;
    float Pfast;                        // single(0.5*log2(P-1) - 1.5)
    // f = f_max - min{ j : T <= theta[j] } where T = sum ceil(|x| 2^(15-e))^2 is the
    // exact integer behind S = T 2^-30 in f = floor(P'_fast - max(1, 0.51 log2 S)).
    int32_t f_max, levels;
    uint64_t theta[kMaxLevels];
    // Accurate mode (Section 4.2): P'_accu = single(0.5*log2(P-1) - 0.5) and the same kind of
    // table for f = floor(P'_accu - 0.51 log2 c) over the integer c = max entry of a row or
    // column of Abar*Bbar (summed over K ranges), 1 <= c <= 2^32: f = accu_f_max - min{ j : c <= accu_theta[j] }.
    float Paccu;
    int32_t accu_f_max, accu_levels;
    uint64_t accu_theta[kMaxLevels];
};

// Built on first use, cached for the life of the process.  n must be in 2..20.
const Table &table(int n, bool is_double);

}  // namespace oz2
