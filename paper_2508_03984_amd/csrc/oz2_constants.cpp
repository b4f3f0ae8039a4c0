// Host-side table of the constants of Section 4.1 ("Determination of
// Constants") for N = 2..20 moduli, computed once with a small fixed-width
// unsigned integer class (the product of 20 moduli needs 156 bits).
#include "oz2_constants.hpp"

#include <cmath>
#include <cstring>
#include <mutex>

namespace oz2 {
namespace {

// 320-bit unsigned integer, little-endian 64-bit limbs.
struct Wide {
    static constexpr int L = 5;
    uint64_t w[L] = {0, 0, 0, 0, 0};

    static Wide from_u64(uint64_t v) { Wide r; r.w[0] = v; return r; }

    // exact for integral d >= 0 below 2^320
    static Wide from_double(double d) {
        int ex;
        double m = std::frexp(d, &ex);                    // d = m * 2^ex, m in [0.5, 1)
        uint64_t mant = (uint64_t)std::ldexp(m, 53);
        Wide r = from_u64(mant);
        int sh = ex - 53;
        if (sh >= 0) return r.shl(sh);
        return r.shr(-sh);
    }

    bool is_zero() const { for (int i = 0; i < L; ++i) if (w[i]) return false; return true; }

    int bit_length() const {
        for (int i = L - 1; i >= 0; --i)
            if (w[i]) return 64 * i + 64 - __builtin_clzll(w[i]);
        return 0;
    }

    bool bit(int i) const { return i >= 0 && i < 64 * L && ((w[i / 64] >> (i % 64)) & 1u); }

    bool any_bit_below(int i) const {                     // any of bits [0, i) set?
        for (int b = 0; b < i && b < 64 * L; ++b) if (bit(b)) return true;
        return false;
    }

    Wide shl(int s) const {
        Wide r;
        for (int i = 0; i < 64 * L - s; ++i) if (bit(i)) r.w[(i + s) / 64] |= 1ull << ((i + s) % 64);
        return r;
    }
    Wide shr(int s) const {
        Wide r;
        for (int i = s; i < 64 * L; ++i) if (bit(i)) r.w[(i - s) / 64] |= 1ull << ((i - s) % 64);
        return r;
    }

    Wide mul_u64(uint64_t m) const {
        Wide r;
        unsigned __int128 carry = 0;
        for (int i = 0; i < L; ++i) {
            unsigned __int128 t = (unsigned __int128)w[i] * m + carry;
            r.w[i] = (uint64_t)t;
            carry = t >> 64;
        }
        return r;
    }

    // quotient; remainder through *rem
    Wide div_u32(uint32_t d, uint32_t *rem = nullptr) const {
        Wide q;
        unsigned __int128 r = 0;
        for (int i = L - 1; i >= 0; --i) {
            unsigned __int128 cur = (r << 64) | w[i];
            q.w[i] = (uint64_t)(cur / d);
            r = cur % d;
        }
        if (rem) *rem = (uint32_t)r;
        return q;
    }

    static int cmp(const Wide &a, const Wide &b) {
        for (int i = L - 1; i >= 0; --i) {
            if (a.w[i] < b.w[i]) return -1;
            if (a.w[i] > b.w[i]) return 1;
        }
        return 0;
    }

    // a - b, requires a >= b
    static Wide sub(const Wide &a, const Wide &b) {
        Wide r;
        unsigned borrow = 0;
        for (int i = 0; i < L; ++i) {
            unsigned __int128 t = (unsigned __int128)a.w[i] - b.w[i] - borrow;
            r.w[i] = (uint64_t)t;
            borrow = (t >> 64) ? 1u : 0u;
        }
        return r;
    }

    static Wide add(const Wide &a, const Wide &b) {
        Wide r;
        unsigned __int128 carry = 0;
        for (int i = 0; i < L; ++i) {
            unsigned __int128 t = (unsigned __int128)a.w[i] + b.w[i] + carry;
            r.w[i] = (uint64_t)t;
            carry = t >> 64;
        }
        return r;
    }

    // round to nearest double, ties to even
    double to_double() const {
        int bl = bit_length();
        if (bl <= 53) return (double)w[0];
        int cut = bl - 53;
        uint64_t mant = shr(cut).w[0];
        bool half = bit(cut - 1);
        bool sticky = any_bit_below(cut - 1);
        if (half && (sticky || (mant & 1))) ++mant;       // may become 2^53: still exact below
        return std::ldexp((double)mant, cut);
    }

    // keep the leading `bits` bits, clear the rest
    Wide keep_top(int bits) const {
        int cut = bit_length() - bits;
        if (cut <= 0) return *this;
        return shr(cut).shl(cut);
    }
};

// Greedy choice of Section 4.1: from 256 downwards, keep what is coprime to all kept so far.
void pick_moduli(int32_t *out, int count) {
    int have = 0;
    for (int c = 256; c >= 2 && have < count; --c) {
        bool ok = true;
        for (int i = 0; i < have && ok; ++i) {
            int a = c, b = out[i];
            while (b) { int t = a % b; a = b; b = t; }
            ok = (a == 1);
        }
        if (ok) out[have++] = c;
    }
}

int ceil_log2(int n) { int r = 0; while ((1 << r) < n) ++r; return r; }

double log2_wide(const Wide &x) {
    int bl = x.bit_length();
    int cut = bl > 64 ? bl - 64 : 0;
    long double top = (long double)x.shr(cut).w[0];
    return (double)(log2l(top) + (long double)cut);
}

// double nearest to 1/P: start from the FP64 quotient and correct it with exact
// integer comparisons (2M-1) * P <= 2^(1-E) <= (2M+1) * P for x = M * 2^E.
double inverse_rn(const Wide &P) {
    double x = 1.0 / P.to_double();
    for (int it = 0; it < 4; ++it) {
        int ex;
        double m = std::frexp(x, &ex);
        uint64_t M = (uint64_t)std::ldexp(m, 53);
        int E = ex - 53;                                    // x = M * 2^E, E < 0
        Wide one = Wide::from_u64(1).shl(1 - E);            // 2^(1-E)
        Wide lo = P.mul_u64(2 * M - 1), hi = P.mul_u64(2 * M + 1);
        if (Wide::cmp(lo, one) > 0) x = std::nextafter(x, 0.0);
        else if (Wide::cmp(hi, one) < 0) x = std::nextafter(x, 1.0);
        else break;
    }
    return x;
}

// f as a function of the integer T (Section 4.2, see the header of this module).
int32_t level_of(uint64_t T, double Pfast) {
    double S = std::ldexp((double)T, -30);
    return (int32_t)std::floor(Pfast - std::fmax(1.0, 0.51 * std::log2(S)));
}

int32_t accu_level_of(uint64_t c, double Paccu) {
    return (int32_t)std::floor(Paccu - 0.51 * std::log2((double)c));
}

Table build(int n, bool is_double) {
    Table t;
    std::memset(&t, 0, sizeof(t));
    t.n = n;
    pick_moduli(t.p, n);

    Wide P = Wide::from_u64(1);
    for (int i = 0; i < n; ++i) P = P.mul_u64((uint64_t)t.p[i]);

    Wide w[kMaxModuli];
    int wmax_log = 0;
    for (int i = 0; i < n; ++i) {
        uint32_t pi = (uint32_t)t.p[i];
        Wide rest = P.div_u32(pi);                          // P / p_i
        uint32_t r;
        rest.div_u32(pi, &r);                               // (P / p_i) mod p_i
        uint32_t q = 1;
        while ((uint64_t)q * r % pi != 1) ++q;              // modular inverse by search
        w[i] = rest.mul_u64(q);
        wmax_log = std::max(wmax_log, w[i].bit_length() - 1);
        t.pinv_prime[i] = (uint32_t)((1ull << 32) / pi - 1);
        t.pinv[i] = 1.0 / (double)pi;
    }

    t.P1 = P.to_double();
    t.Pinv = inverse_rn(P);
    t.Pfast = (float)(0.5 * log2_wide(Wide::sub(P, Wide::from_u64(1))) - 1.5);

    if (is_double) {
        Wide P1w = Wide::from_double(t.P1);
        t.P2 = Wide::cmp(P, P1w) >= 0 ? Wide::sub(P, P1w).to_double()
                                      : -Wide::sub(P1w, P).to_double();
        for (int i = 0; i < n; ++i) {
            int beta = 53 - 8 - ceil_log2(n) + (w[i].bit_length() - 1) - wmax_log;
            Wide hi = w[i].keep_top(beta);
            t.s1[i] = hi.to_double();                       // exact: <= 45 significant bits
            t.s2[i] = Wide::sub(w[i], hi).to_double();
        }
    } else {
        t.P2 = 0.0;
        for (int i = 0; i < n; ++i) { t.s1[i] = w[i].to_double(); t.s2[i] = 0.0; }
    }

    // Shift table: theta[j] = largest T in [2^30, 2^52] with level_of(T) >= f_max - j
    // (T <= 2^32 k, and k <= 2^20 is the longest supported contraction).
    const uint64_t Tmin = 1ull << 30, Tmax = 1ull << 52;
    double Pf = (double)t.Pfast;
    t.f_max = level_of(Tmin, Pf);
    int32_t f_min = level_of(Tmax, Pf);
    t.levels = t.f_max - f_min + 1;
    for (int j = 0; j < t.levels && j < kMaxLevels; ++j) {
        int32_t want = t.f_max - j;
        uint64_t lo = Tmin, hi = Tmax;                      // level_of(lo) >= want always
        while (lo < hi) {
            uint64_t mid = lo + (hi - lo + 1) / 2;
            if (level_of(mid, Pf) >= want) lo = mid; else hi = mid - 1;
        }
        t.theta[j] = lo;
    }
    if (t.levels > kMaxLevels) t.levels = -1;               // cannot happen for N <= 20

    // Accurate-mode table over c in [1, 2^32]: a K range of 2^17 gives entries of at most
    // 2^17 * 64 * 64 = 2^29, and up to 8 ranges are summed.
    t.Paccu = (float)(0.5 * log2_wide(Wide::sub(P, Wide::from_u64(1))) - 0.5);
    const uint64_t Cmax = 1ull << 32;
    double Pa = (double)t.Paccu;
    t.accu_f_max = accu_level_of(1, Pa);
    t.accu_levels = t.accu_f_max - accu_level_of(Cmax, Pa) + 1;
    for (int j = 0; j < t.accu_levels && j < kMaxLevels; ++j) {
        int32_t want = t.accu_f_max - j;
        uint64_t lo = 1, hi = Cmax;
        while (lo < hi) {
            uint64_t mid = lo + (hi - lo + 1) / 2;
            if (accu_level_of(mid, Pa) >= want) lo = mid; else hi = mid - 1;
        }
        t.accu_theta[j] = lo;
    }
    if (t.accu_levels > kMaxLevels) t.accu_levels = -1;
    return t;
}

}  // namespace

const Table &table(int n, bool is_double) {
    static Table cache[2][kMaxModuli + 1];
    static bool ready[2][kMaxModuli + 1];
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    int d = is_double ? 1 : 0;
    if (!ready[d][n]) { cache[d][n] = build(n, is_double); ready[d][n] = true; }
    return cache[d][n];
}

}  // namespace oz2
