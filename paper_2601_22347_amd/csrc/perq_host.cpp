// Host side of the PeRQ library: status strings, Algorithm 1 (mass diffusion), the permutation
// validator and the base matrices of the non-power-of-two rotation.  No device code here.
#include "perq.h"
#include "perq_base.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <queue>
#include <utility>
#include <vector>

extern "C" const char* perq_status_string(perq_status_t status) {
    switch (status) {
        case PERQ_OK: return "PERQ_OK";
        case PERQ_ERR_INVALID_ARG: return "PERQ_ERR_INVALID_ARG";
        case PERQ_ERR_UNSUPPORTED: return "PERQ_ERR_UNSUPPORTED";
        case PERQ_ERR_LAUNCH: return "PERQ_ERR_LAUNCH";
    }
    return "PERQ_ERR_UNKNOWN";
}

// Algorithm 1.  The argmin over not-yet-full blocks of the accumulated block mass is served by
// a binary heap keyed on (mass, block index); a block that fills up is simply not pushed back,
// which is the algorithm's "drop j* from the valid set".  Lexicographic keys give the
// lowest-index block among equal masses, the stable sort gives the lower channel among equal
// means -- the two tie rules the paper leaves open.
extern "C" perq_status_t perq_massdiff_perm(const float* colabs_mean, int32_t d, int32_t b,
                                            int32_t* perm_out) {
    if (colabs_mean == nullptr || perm_out == nullptr) return PERQ_ERR_INVALID_ARG;
    if (d <= 0 || b <= 0 || d % b != 0) return PERQ_ERR_INVALID_ARG;
    for (int32_t i = 0; i < d; ++i)
        if (!std::isfinite(colabs_mean[i]) || colabs_mean[i] < 0.0f) return PERQ_ERR_INVALID_ARG;

    const int32_t n = d / b;
    std::vector<int32_t> order(d);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
        return colabs_mean[x] > colabs_mean[y];
    });

    using Key = std::pair<double, int32_t>;   // (accumulated mass L_j, block j)
    std::priority_queue<Key, std::vector<Key>, std::greater<Key>> valid;
    for (int32_t j = 0; j < n; ++j) valid.emplace(0.0, j);
    std::vector<int32_t> fill(n, 0);

    for (int32_t i : order) {
        Key top = valid.top();
        valid.pop();
        const int32_t j = top.second;
        perm_out[static_cast<int64_t>(j) * b + fill[j]] = i;
        if (++fill[j] < b) valid.emplace(top.first + static_cast<double>(colabs_mean[i]), j);
    }
    return PERQ_OK;
}

// The two other calibrated permutations of the ablation (Appendix C, "Permutations").
static bool stat_ok(const float* stat, int32_t d) {
    for (int32_t i = 0; i < d; ++i)
        if (!std::isfinite(stat[i]) || stat[i] < 0.0f) return false;
    return true;
}

extern "C" perq_status_t perq_perm_sorted(const float* stat, int32_t d, int32_t* perm_out) {
    if (stat == nullptr || perm_out == nullptr || d <= 0) return PERQ_ERR_INVALID_ARG;
    if (!stat_ok(stat, d)) return PERQ_ERR_INVALID_ARG;
    std::iota(perm_out, perm_out + d, 0);
    std::stable_sort(perm_out, perm_out + d, [&](int32_t x, int32_t y) { return stat[x] > stat[y]; });
    return PERQ_OK;
}

extern "C" perq_status_t perq_perm_zigzag(const float* stat, int32_t d, int32_t b, int32_t* perm_out) {
    if (stat == nullptr || perm_out == nullptr) return PERQ_ERR_INVALID_ARG;
    if (d <= 0 || b <= 0 || d % b != 0) return PERQ_ERR_INVALID_ARG;
    if (!stat_ok(stat, d)) return PERQ_ERR_INVALID_ARG;
    const int32_t n = d / b;
    std::vector<int32_t> order(d);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return stat[x] > stat[y]; });
    // round k of n ranks fills slot k of every block, left to right on even rounds, right to left on odd
    for (int32_t r = 0; r < d; ++r) {
        const int32_t round = r / n, pos = r % n;
        const int32_t blk = (round & 1) ? n - 1 - pos : pos;
        perm_out[static_cast<int64_t>(blk) * b + round] = order[r];
    }
    return PERQ_OK;
}

extern "C" perq_status_t perq_perm_random(int32_t d, uint64_t seed, int32_t* perm_out) {
    if (perm_out == nullptr || d <= 0) return PERQ_ERR_INVALID_ARG;
    for (int32_t i = 0; i < d; ++i) perm_out[i] = i;
    uint64_t state = seed;
    for (int32_t i = d - 1; i > 0; --i) {
        // SplitMix64: next state, then two xor-shift-multiply rounds
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        const uint64_t j = (uint64_t)(((unsigned __int128)z * (uint64_t)(i + 1)) >> 64);
        std::swap(perm_out[i], perm_out[j]);
    }
    return PERQ_OK;
}

extern "C" perq_status_t perq_perm_validate(const int32_t* perm_host, int32_t d) {
    if (perm_host == nullptr || d <= 0) return PERQ_ERR_INVALID_ARG;
    std::vector<uint8_t> seen(d, 0);
    for (int32_t i = 0; i < d; ++i) {
        const int32_t p = perm_host[i];
        if (p < 0 || p >= d || seen[p]) return PERQ_ERR_INVALID_ARG;
        seen[p] = 1;
    }
    return PERQ_OK;
}

// ---- base matrices of the non-power-of-two rotation (Appendix A.1) -----------------------------
namespace perq {
namespace {

bool prime(int32_t q) {
    if (q < 2) return false;
    for (int32_t f = 2; (int64_t)f * f <= q; ++f)
        if (q % f == 0) return false;
    return true;
}

// Legendre symbol of v modulo the odd prime q by Euler's criterion: v^((q-1)/2) mod q.
int legendre(int32_t v, int32_t q) {
    v %= q;
    if (v < 0) v += q;
    if (v == 0) return 0;
    int64_t acc = 1, base = v;
    for (int32_t e = (q - 1) / 2; e > 0; e >>= 1) {
        if (e & 1) acc = acc * base % q;
        base = base * base % q;
    }
    return acc == 1 ? 1 : -1;
}

}  // namespace

int hadamard_base_kind(int32_t m) {
    if (m < 12 || m % 8 != 4) return 0;      // m = 4t with t odd and above 1 (a power of two has Sylvester's matrix)
    if (prime(m - 1) && (m - 1) % 4 == 3) return 1;
    if (prime(m / 2 - 1) && (m / 2 - 1) % 4 == 1) return 2;
    return 0;
}

int hadamard_base_entry(int32_t m, int kind, int32_t r, int32_t c) {
    if (kind == 1) {
        // I + S, S = [[0, 1^T], [-1, Q]], Q[i][j] = chi(i - j) over Z_(m-1)
        if (r == c) return 1;
        if (r == 0) return 1;
        if (c == 0) return -1;
        return legendre(r - c, m - 1);
    }
    // S = [[0, 1^T], [1, Q]] over Z_(m/2-1); a zero of S becomes [[1,-1],[-1,-1]], an entry e
    // becomes e [[1,1],[1,-1]]
    const int32_t R = r >> 1, C = c >> 1, q = m / 2 - 1;
    const int rr = r & 1, cc = c & 1;
    int e;
    if (R == C) e = 0;
    else if (R == 0 || C == 0) e = 1;
    else e = legendre(R - C, q);
    if (e == 0) return (rr == 0 && cc == 0) ? 1 : -1;
    return (rr == 1 && cc == 1) ? -e : e;
}

}  // namespace perq

extern "C" perq_status_t perq_hadamard_base(int32_t m, int8_t* out) {
    if (out == nullptr) return PERQ_ERR_INVALID_ARG;
    const int kind = perq::hadamard_base_kind(m);
    if (kind == 0) return PERQ_ERR_INVALID_ARG;
    for (int32_t r = 0; r < m; ++r)
        for (int32_t c = 0; c < m; ++c) out[(int64_t)r * m + c] = (int8_t)perq::hadamard_base_entry(m, kind, r, c);
    return PERQ_OK;
}
