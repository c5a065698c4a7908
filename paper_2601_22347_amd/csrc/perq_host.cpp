// Host side of the PeRQ library: status strings, Algorithm 1 (mass diffusion), the permutation
// validator and the base matrices of the non-power-of-two rotation.  No device code here.
#include "perq.h"
#include "perq_base.h"
#include "perq_layout.h"
#include "perq_schedule.h"

#include <algorithm>
#include <array>
#include <climits>
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
        case PERQ_ERR_INTERNAL: return "PERQ_ERR_INTERNAL";
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


// ---- a permutation arranged for the operand gather of the matrix-core kernel ---------------------
// With a permutation every operand element is a 2-byte LDS read at an address of its own; one read
// instruction fetches, for the 32 lanes of each half-wave, one position each (perq_layout.h), and on
// arbitrary addresses several lanes meet in one of the 32 four-byte banks.  Which channels a block
// holds is Algorithm 1's result and fixes the block masses, hence the bound of Proposition 2; the
// order inside a block is free (P is merged into the weights either way).  The routine below keeps
// every block's set and orders it so that the lanes of a read instruction meet different banks.
namespace {

struct GatherShape {
    bool ok;        // the shape runs on the matrix-core kernel with the element-wise gather
    bool high_k;    // b >= 1024
    int tiles;
};

GatherShape gather_shape(int32_t d, int32_t b) {
    GatherShape s{false, false, 0};
    if (d < 4096 || d > PERQ_MAX_D || d % 512 != 0) return s;
    if (b < 16 || b > 4096 || (b & (b - 1)) != 0 || d % b != 0) return s;
    s.ok = true;
    s.high_k = b >= 1024;
    s.tiles = (d + 4095) / 4096;
    return s;
}

inline int bank_of(int32_t channel) { return (int)((perq::layout::channel_offset((uint32_t)channel) >> 2) & 31u); }

// Calls visit(positions, n) once per read instruction and half-wave with the positions (in the row)
// that its lanes fetch; lanes past the end of a ragged last tile are left out.
template <class F>
void for_each_read(int32_t d, const GatherShape& s, F&& visit) {
    int32_t pos[32];
    for (int t = 0; t < s.tiles; ++t) {
        const int32_t tile_len = std::min<int32_t>(4096, d - 4096 * t);
        for (uint32_t f = 0; f < 8; ++f)
            for (uint32_t e = 0; e < 8; ++e)
                for (uint32_t h = 0; h < 2; ++h) {
                    int n = 0;
                    for (uint32_t l = 0; l < 32; ++l) {
                        const int32_t in_tile = (int32_t)perq::layout::gather_pos(s.high_k, l, h, f, e);
                        if (in_tile < tile_len) pos[n++] = 4096 * t + in_tile;
                    }
                    if (n > 0) visit(pos, n);
                }
    }
}

}  // namespace

namespace {

// sum over the read instructions (per half-wave) of the largest number of lanes that meet in one bank
// on different words; *reads = number of such instructions
int64_t gather_passes(const int32_t* perm, int32_t d, const GatherShape& s, int64_t* reads) {
    int64_t total = 0, count = 0;
    for_each_read(d, s, [&](const int32_t* pos, int n) {
        // lanes in one bank are served one after another unless they want the same four bytes
        int load[32] = {0};
        int32_t seen[32][32];
        for (int i = 0; i < n; ++i) {
            const uint32_t off = perq::layout::channel_offset((uint32_t)perm[pos[i]]);
            const int bank = (int)((off >> 2) & 31u);
            const int32_t word = (int32_t)(off >> 2);
            bool dup = false;
            for (int k = 0; k < load[bank]; ++k) dup = dup || seen[bank][k] == word;
            if (!dup) seen[bank][load[bank]++] = word;
        }
        total += *std::max_element(load, load + 32);
        ++count;
    });
    if (reads != nullptr) *reads = count;
    return total;
}

}  // namespace

extern "C" perq_status_t perq_perm_gather_cost(const int32_t* perm, int32_t d, int32_t b, int64_t* passes,
                                               int64_t* reads) {
    if (perm == nullptr || passes == nullptr || reads == nullptr || d <= 0) return PERQ_ERR_INVALID_ARG;
    if (perq_perm_validate(perm, d) != PERQ_OK) return PERQ_ERR_INVALID_ARG;
    const GatherShape s = gather_shape(d, b);
    if (!s.ok) return PERQ_ERR_UNSUPPORTED;
    *passes = gather_passes(perm, d, s, reads);
    return PERQ_OK;
}

extern "C" perq_status_t perq_perm_arrange(const int32_t* perm, int32_t d, int32_t b, int32_t head, int32_t* perm_out) {
    if (perm == nullptr || perm_out == nullptr || d <= 0 || b <= 0 || d % b != 0) return PERQ_ERR_INVALID_ARG;
    if (head < 0) head = b >= 512 ? 64 : 0;
    if (head > b) return PERQ_ERR_INVALID_ARG;
    if (perq_perm_validate(perm, d) != PERQ_OK) return PERQ_ERR_INVALID_ARG;
    const GatherShape s = gather_shape(d, b);
    if (!s.ok) {                       // no such gather for this shape: nothing to gain, nothing changed
        std::copy(perm, perm + d, perm_out);
        return PERQ_OK;
    }
    const int32_t nblocks = d / b;
    // Which block sits where in the row is as free as the order inside a block.  The lanes of a read
    // fetch from the blocks of one "bin": a 4096-wide tile, or for b < 128 in the low-K modes the
    // blocks of a tile with the same index modulo 128 / b (block k * (128 / b) + m of the tile is the
    // m-th of lane k).  A read can only be free of conflicts if the channels of its bin are spread
    // evenly over the banks (a bin holds an arbitrary subset of the d channels), so the blocks are
    // first dealt to the bins with that in mind: each to the bin whose fullest bank it raises least
    // above the level of an even spread, then pairs of blocks are exchanged between bins while that
    // lowers the sum of the bins' fullest banks.  Inside a bin the blocks keep their order.
    std::vector<int32_t> block_at(nblocks);                 // block_at[place] = block of perm
    {
        std::vector<std::array<int32_t, 32>> hist(nblocks);
        for (int32_t j = 0; j < nblocks; ++j) {
            hist[j].fill(0);
            for (int32_t i = 0; i < b; ++i) ++hist[j][bank_of(perm[(size_t)j * b + i])];
        }
        const int ndom = (!s.high_k && b < 128) ? 128 / b : 1;
        const int bins = s.tiles * ndom;
        std::vector<int32_t> cap(bins), bin_of(nblocks, -1);
        std::vector<std::array<int32_t, 32>> total(bins);
        std::vector<int32_t> filled(bins, 0);
        for (int q = 0; q < bins; ++q) {
            cap[q] = std::min<int32_t>(4096, d - 4096 * (q / ndom)) / b / ndom;
            total[q].fill(0);
        }
        auto peak_with = [&](int q, int32_t add, int32_t drop) {
            int32_t m = 0;
            for (int k = 0; k < 32; ++k)
                m = std::max(m, total[q][k] + (add >= 0 ? hist[add][k] : 0) - (drop >= 0 ? hist[drop][k] : 0));
            return m;
        };
        if (bins > 1 && cap[0] > 1) {
            for (int32_t j = 0; j < nblocks; ++j) {
                int best = -1;
                int64_t best_cost = 0;
                for (int q = 0; q < bins; ++q) {
                    if (filled[q] == cap[q]) continue;
                    // excess of the fullest bank over an even spread, in units of 1/32 channel
                    const int64_t cost = (int64_t)peak_with(q, j, -1) * 32 - (int64_t)(filled[q] + 1) * b;
                    if (best < 0 || cost < best_cost || (cost == best_cost && cap[q] - filled[q] > cap[best] - filled[best])) {
                        best = q;
                        best_cost = cost;
                    }
                }
                bin_of[j] = best;
                ++filled[best];
                for (int k = 0; k < 32; ++k) total[best][k] += hist[j][k];
            }
            const int passes = nblocks > 1024 ? 1 : 4;      // (pairs of blocks: quadratic)
            for (int pass = 0; pass < passes; ++pass) {
                bool changed = false;
                for (int32_t x = 0; x < nblocks; ++x)
                    for (int32_t y = x + 1; y < nblocks; ++y) {
                        const int qx = bin_of[x], qy = bin_of[y];
                        if (qx == qy) continue;
                        const int32_t before = peak_with(qx, -1, -1) + peak_with(qy, -1, -1);
                        const int32_t after = peak_with(qx, y, x) + peak_with(qy, x, y);
                        if (after < before) {
                            for (int k = 0; k < 32; ++k) {
                                total[qx][k] += hist[y][k] - hist[x][k];
                                total[qy][k] += hist[x][k] - hist[y][k];
                            }
                            std::swap(bin_of[x], bin_of[y]);
                            changed = true;
                        }
                    }
                if (!changed) break;
            }
            std::vector<int32_t> next(bins, 0);             // blocks placed so far, per bin
            int32_t tile_first = 0;                         // first block place of the tile
            for (int t = 0; t < s.tiles; ++t) {
                for (int32_t j = 0; j < nblocks; ++j) {
                    const int q = bin_of[j];
                    if (q / ndom != t) continue;
                    block_at[tile_first + next[q] * ndom + q % ndom] = j;
                    ++next[q];
                }
                tile_first += std::min<int32_t>(4096, d - 4096 * t) / b;
            }
        } else {
            std::iota(block_at.begin(), block_at.end(), 0);
        }
    }
    // the channels of every block, by bank (ascending inside a bank: the result is deterministic)
    // The first `head` positions of every block keep the channels they were given (each is a pool of
    // its own with one channel); the others share the pool of their block.
    std::vector<int32_t> pool_of(d);
    {
        int32_t next_pool = nblocks;
        for (int32_t pos = 0; pos < d; ++pos) pool_of[pos] = pos % b < head ? next_pool++ : pos / b;
    }
    std::vector<std::vector<int32_t>> pool((size_t)(nblocks + (size_t)nblocks * head) * 32);
    for (int32_t j = 0; j < nblocks; ++j) {
        const int32_t* src = perm + (size_t)block_at[j] * b;
        for (int32_t i = 0; i < head; ++i) pool[(size_t)pool_of[j * b + i] * 32 + bank_of(src[i])].push_back(src[i]);
        std::vector<int32_t> chans(src + head, src + b);
        std::sort(chans.begin(), chans.end(), std::greater<int32_t>());
        for (int32_t c : chans) pool[(size_t)j * 32 + bank_of(c)].push_back(c);     // taken from the back
    }
    std::vector<int32_t> arranged(d);
    bool broken = false;
    for_each_read(d, s, [&](const int32_t* pos, int n) {
        if (broken) return;
        // a matching of lanes to banks (Kuhn's augmenting paths), lanes with the fewest banks on
        // offer first, banks tried in the order of what the lane's block still holds most of
        int order[32], lane_bank[32], bank_lane[32];
        std::vector<int> adj[32];
        for (int i = 0; i < n; ++i) {
            const size_t blk = (size_t)pool_of[pos[i]] * 32;
            for (int k = 0; k < 32; ++k)
                if (!pool[blk + k].empty()) adj[i].push_back(k);
            std::stable_sort(adj[i].begin(), adj[i].end(), [&](int x, int y) { return pool[blk + x].size() > pool[blk + y].size(); });
            order[i] = i;
            lane_bank[i] = -1;
        }
        std::fill(bank_lane, bank_lane + 32, -1);
        std::stable_sort(order, order + n, [&](int x, int y) { return adj[x].size() < adj[y].size(); });
        // (for the lanes left over below) two lanes of one block may not both count on the last channel of a bank
        auto free_in = [&](int lane, int bank) {
            const size_t blk = (size_t)pool_of[pos[lane]] * 32;
            size_t taken = 0;
            for (int i = 0; i < n; ++i)
                if (i != lane && lane_bank[i] == bank && (size_t)pool_of[pos[i]] * 32 == blk) ++taken;
            return pool[blk + bank].size() > taken;
        };
        bool visited[32];
        auto augment = [&](auto&& self, int lane) -> bool {
            for (int k : adj[lane]) {
                if (visited[k]) continue;      // (a bank holds one lane here, so its pool is never short)
                visited[k] = true;
                if (bank_lane[k] < 0 || self(self, bank_lane[k])) {
                    bank_lane[k] = lane;
                    lane_bank[lane] = k;
                    return true;
                }
            }
            return false;
        };
        for (int q = 0; q < n; ++q) {
            std::fill(visited, visited + 32, false);
            augment(augment, order[q]);
        }
        // lanes left over share a bank: the least loaded one their block can still serve
        int load[32];
        for (int k = 0; k < 32; ++k) load[k] = bank_lane[k] >= 0 ? 1 : 0;
        for (int q = 0; q < n; ++q) {
            const int lane = order[q];
            if (lane_bank[lane] >= 0) continue;
            int best = -1;
            for (int k : adj[lane])
                if (free_in(lane, k) && (best < 0 || load[k] < load[best])) best = k;
            if (best < 0) {            // cannot happen: a block holds as many channels as positions are left
                broken = true;
                return;
            }
            lane_bank[lane] = best;
            ++load[best];
        }
        for (int i = 0; i < n; ++i) {
            std::vector<int32_t>& from = pool[(size_t)pool_of[pos[i]] * 32 + lane_bank[i]];
            arranged[pos[i]] = from.back();
            from.pop_back();
        }
    });
    if (broken) return PERQ_ERR_INTERNAL;
    // never worse than what was given (heads that stay in place can meet in one bank when the given
    // order is regular, e.g. blocks of consecutive channels)
    if (gather_passes(arranged.data(), d, s, nullptr) >= gather_passes(perm, d, s, nullptr))
        std::copy(perm, perm + d, arranged.begin());
    std::copy(arranged.begin(), arranged.end(), perm_out);
    return PERQ_OK;
}

// ---- placement of a row's 16-byte granules in LDS for a given permutation ----------------------------
// The kernel stages a row with direct-to-LDS loads of 16 bytes per lane, 64 consecutive slots per
// instruction, and is free in which granule of the row a lane fetches.  Eight consecutive lanes fetch
// the eight granules of one 128-byte line of the row, in any order: the loads stay as coalesced as
// they are with the fixed layout.  The bank of a channel is 4 * (slot % 8) + (channel % 8) / 2, so the
// order decides, per granule, which group of four banks its eight channels land in.  The fixed
// swizzle of perq_layout.h spreads the identity and strided patterns; for an arbitrary permutation the
// 32 lanes of a read meet at random (3.2 - 3.5 passes per read).  Here the order inside every line is
// chosen for the permutation at hand.  Lanes whose channels share the pattern (channel % 8) / 2 can
// only be told apart by the eight groups, so a read whose 32 channels hold more than eight of one
// pattern keeps two passes.  The two 64-byte halves of a line stay halves (four neighbouring lanes fetch
// one of them); about 2.3 passes per read are reached.
namespace {

struct PlacementProblem {
    int32_t d;
    int32_t n_granules;
    std::vector<std::vector<std::pair<int32_t, uint8_t>>> member;   // per granule: (read, word % 4) of its words
    int32_t n_reads;
};

PlacementProblem placement_problem(const int32_t* perm, int32_t d, const GatherShape& s) {
    PlacementProblem pb;
    pb.d = d;
    pb.n_granules = d / 8;
    pb.member.assign((size_t)pb.n_granules, {});
    int32_t r = 0;
    for_each_read(d, s, [&](const int32_t* pos, int n) {
        int32_t words[32];
        int nw = 0;
        for (int i = 0; i < n; ++i) {
            const int32_t w = perm[pos[i]] >> 1;
            bool dup = false;
            for (int k = 0; k < nw; ++k) dup = dup || words[k] == w;
            if (!dup) words[nw++] = w;
        }
        for (int k = 0; k < nw; ++k) pb.member[(size_t)(words[k] >> 2)].emplace_back(r, (uint8_t)(words[k] & 3));
        ++r;
    });
    pb.n_reads = r;
    return pb;
}

// sum over the reads of the fullest bank, for group[granule] in 0..7
int64_t placement_passes(const PlacementProblem& pb, const std::vector<uint8_t>& group) {
    std::vector<std::array<uint8_t, 32>> load((size_t)pb.n_reads);
    for (auto& l : load) l.fill(0);
    for (int32_t g = 0; g < pb.n_granules; ++g)
        for (const auto& m : pb.member[(size_t)g]) ++load[(size_t)m.first][4 * group[(size_t)g] + m.second];
    int64_t total = 0;
    for (const auto& l : load) total += *std::max_element(l.begin(), l.end());
    return total;
}

}  // namespace

// The prepared form of a permutation: [int32 place of the channel of every position, d entries]
// [uint16 granule of every slot, d / 8 entries] [uint16 operand offsets in the kernel's lane order, one
// table for b <= 512 and one for b >= 1024, each tiles x 8 fragments x 64 lanes x 8 elements].
namespace {
size_t prepared_lane_tables_at(int32_t d) { return (size_t)d * sizeof(int32_t) + (size_t)(d / 8) * sizeof(uint16_t); }
size_t lane_table_entries(int32_t d) { return (size_t)((d + 4095) / 4096) * 4096; }

// Byte offset inside the staged row of the operand that read (f, e) of lane l fetches, for every tile,
// fragment, lane and element: what the kernel otherwise works out from `perm` at the start of every
// launch.  0xFFFF (no offset is odd) marks positions past the end of a ragged last tile.
void fill_lane_tables(const int32_t* perm, int32_t d, const std::vector<int32_t>& slot_of_granule, uint16_t* tables) {
    const bool placed = perq::layout::placement_applies(d);
    const int tiles = (d + 4095) / 4096;
    for (int mode = 0; mode < 2; ++mode) {
        uint16_t* tab = tables + (size_t)mode * lane_table_entries(d);
        for (int t = 0; t < tiles; ++t)
            for (uint32_t f = 0; f < 8; ++f)
                for (uint32_t lane = 0; lane < 64; ++lane)
                    for (uint32_t e = 0; e < 8; ++e) {
                        const int64_t pos = 4096 * (int64_t)t + perq::layout::gather_pos(mode == 1, lane & 31u, lane >> 5, f, e);
                        uint16_t off = 0xFFFFu;
                        if (pos < d) {
                            const uint32_t a = (uint32_t)perm[pos];
                            off = placed ? (uint16_t)(((uint32_t)slot_of_granule[a >> 3] << 4) | ((a & 7u) << 1))
                                         : (uint16_t)perq::layout::channel_offset(a);
                        }
                        tab[(((size_t)t * 8 + f) * 64 + lane) * 8 + e] = off;
                    }
    }
}
}  // namespace

extern "C" size_t perq_perm_prepared_bytes(int32_t d) {
    if (d <= 0 || d % 8 != 0) return 0;
    return prepared_lane_tables_at(d) + 2 * lane_table_entries(d) * sizeof(uint16_t);
}

extern "C" perq_status_t perq_perm_prepare(const int32_t* perm, int32_t d, int32_t b, void* prepared,
                                           int64_t* passes_before, int64_t* passes_after, int64_t* reads) {
    if (perm == nullptr || prepared == nullptr || d <= 0 || b <= 0) return PERQ_ERR_INVALID_ARG;
    if (perq_perm_validate(perm, d) != PERQ_OK) return PERQ_ERR_INVALID_ARG;
    const GatherShape s = gather_shape(d, b);
    if (!s.ok) return PERQ_ERR_UNSUPPORTED;
    const PlacementProblem pb = placement_problem(perm, d, s);
    const int32_t G = pb.n_granules;                                // (d is a multiple of 512)
    // what the fixed swizzle gives
    std::vector<uint8_t> group((size_t)G);
    for (int32_t g = 0; g < G; ++g) group[(size_t)g] = (uint8_t)(perq::layout::granule_slot((uint32_t)g) & 7u);
    const int64_t before = placement_passes(pb, group);

    // One 128-byte line of the row (8 granules) at a time: its granules take the 8 groups of four banks
    // in some order, the order that costs least given the lines placed so far (an 8 x 8 assignment,
    // solved exactly over subsets).  Cost of a granule in a group: for every read it takes part in,
    // the words already in that bank, and a large penalty where it would raise the read's fullest bank.
    std::vector<std::array<uint8_t, 32>> load((size_t)pb.n_reads);
    for (auto& l : load) l.fill(0);
    uint64_t rng = 0x9E3779B97F4A7C15ull;
    auto next_rand = [&]() {
        rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
        return rng;
    };
    const int32_t n_lines = G / 8;
    std::vector<int32_t> order((size_t)n_lines);
    std::iota(order.begin(), order.end(), 0);
    for (int32_t i = n_lines - 1; i > 0; --i) std::swap(order[(size_t)i], order[(size_t)(next_rand() % (uint64_t)(i + 1))]);
    std::vector<uint8_t> chosen((size_t)G, 0xFF);
    auto put = [&](int32_t g, int q, int sign) {
        for (const auto& m : pb.member[(size_t)g]) load[(size_t)m.first][4 * q + m.second] = (uint8_t)(load[(size_t)m.first][4 * q + m.second] + sign);
    };
    auto place_line = [&](int32_t line) {
        int32_t cost[8][8];
        for (int i = 0; i < 8; ++i) {
            const int32_t g = 8 * line + i;
            for (int q = 0; q < 8; ++q) {
                int32_t c = 0;
                for (const auto& m : pb.member[(size_t)g]) {
                    const auto& l = load[(size_t)m.first];
                    const int here = l[4 * q + m.second];
                    const int top = *std::max_element(l.begin(), l.end());
                    c += here + (here + 1 > top ? 1000 : 0);
                }
                cost[i][q] = c;
            }
        }
        // granule i = popcount(mask) - 1 takes a group in mask; the two halves of the line (64 bytes, what
        // four neighbouring lanes fetch together) stay halves, in either order
        int32_t best_total = INT32_MAX;
        uint8_t best_q[8] = {0, 1, 2, 3, 4, 5, 6, 7};
        for (int swap = 0; swap < 2; ++swap) {
            int32_t best[256];
            int8_t pick[256];
            best[0] = 0;
            for (int mask = 1; mask < 256; ++mask) {
                const int i = __builtin_popcount(mask) - 1;
                best[mask] = INT32_MAX;
                pick[mask] = -1;
                for (int q = 0; q < 8; ++q) {
                    if (!((mask >> q) & 1) || ((q >> 2) != ((i >> 2) ^ swap))) continue;
                    const int32_t prev = best[mask ^ (1 << q)];
                    if (prev == INT32_MAX) continue;
                    const int32_t c = prev + cost[i][q];
                    if (c < best[mask]) { best[mask] = c; pick[mask] = (int8_t)q; }
                }
            }
            if (best[255] < best_total) {
                best_total = best[255];
                int mask = 255;
                for (int i = 7; i >= 0; --i) {
                    const int q = pick[mask];
                    best_q[i] = (uint8_t)q;
                    mask ^= 1 << q;
                }
            }
        }
        for (int i = 0; i < 8; ++i) chosen[(size_t)(8 * line + i)] = best_q[i];
        for (int i = 0; i < 8; ++i) put(8 * line + i, chosen[(size_t)(8 * line + i)], +1);
    };
    for (int32_t line : order) place_line(line);
    int64_t now = 0;
    for (const auto& l : load) now += *std::max_element(l.begin(), l.end());
    for (int sweep = 0; sweep < 4; ++sweep) {
        for (int32_t line : order) {
            for (int i = 0; i < 8; ++i) put(8 * line + i, chosen[(size_t)(8 * line + i)], -1);
            place_line(line);
        }
        int64_t then = 0;
        for (const auto& l : load) then += *std::max_element(l.begin(), l.end());
        if (then >= now) break;
        now = then;
    }
    int64_t after = placement_passes(pb, chosen);
    if (after >= before) {               // never worse than the fixed swizzle
        chosen = group;
        after = before;
    }
    // a granule stays in its line: slot = first slot of the line + its group
    int32_t* place_of_position = static_cast<int32_t*>(prepared);
    uint16_t* granule_of_slot = reinterpret_cast<uint16_t*>(place_of_position + d);
    std::vector<int32_t> slot_of_granule((size_t)G);
    for (int32_t g = 0; g < G; ++g) {
        const int32_t slot = (g & ~7) | chosen[(size_t)g];
        slot_of_granule[(size_t)g] = slot;
        granule_of_slot[slot] = (uint16_t)g;
    }
    std::vector<int32_t> places((size_t)d);               // (perm may be the first part of `prepared`)
    for (int32_t i = 0; i < d; ++i) places[(size_t)i] = slot_of_granule[(size_t)(perm[i] >> 3)] * 8 + (perm[i] & 7);
    std::vector<uint16_t> tables(2 * lane_table_entries(d));
    fill_lane_tables(perm, d, slot_of_granule, tables.data());
    std::copy(places.begin(), places.end(), place_of_position);
    std::copy(tables.begin(), tables.end(), reinterpret_cast<uint16_t*>(static_cast<char*>(prepared) + prepared_lane_tables_at(d)));
    if (passes_before != nullptr) *passes_before = before;
    if (passes_after != nullptr) *passes_after = after;
    if (reads != nullptr) *reads = pb.n_reads;
    return PERQ_OK;
}

extern "C" perq_status_t perq_perm_prepared_validate(const void* prepared, const int32_t* perm, int32_t d) {
    if (prepared == nullptr || perm == nullptr || d <= 0 || d % 512 != 0) return PERQ_ERR_INVALID_ARG;
    if (perq_perm_validate(perm, d) != PERQ_OK) return PERQ_ERR_INVALID_ARG;
    const int32_t G = d / 8;
    const int32_t* place_of_position = static_cast<const int32_t*>(prepared);
    const uint16_t* granule_of_slot = reinterpret_cast<const uint16_t*>(place_of_position + d);
    std::vector<int32_t> slot_of_granule((size_t)G, -1);
    for (int32_t slot = 0; slot < G; ++slot) {
        const int32_t g = granule_of_slot[slot];
        if (g >= G || g / 8 != slot / 8 || slot_of_granule[(size_t)g] >= 0) return PERQ_ERR_INVALID_ARG;
        slot_of_granule[(size_t)g] = slot;
    }
    for (int32_t i = 0; i < d; ++i)
        if (place_of_position[i] != slot_of_granule[(size_t)(perm[i] >> 3)] * 8 + (perm[i] & 7)) return PERQ_ERR_INVALID_ARG;
    std::vector<uint16_t> tables(2 * lane_table_entries(d));
    fill_lane_tables(perm, d, slot_of_granule, tables.data());
    const uint16_t* given = reinterpret_cast<const uint16_t*>(static_cast<const char*>(prepared) + prepared_lane_tables_at(d));
    if (!std::equal(tables.begin(), tables.end(), given)) return PERQ_ERR_INVALID_ARG;
    return PERQ_OK;
}

// Host model of the matrix-core kernel's run-time row schedule, on the kernel's own queue
// arithmetic (perq_schedule.h).  Every worker goes through the kernel's sequence -- two fixed
// units, one ticket drawn ahead per unit, stop at the first ticket past the queue's end, the
// drawer of the last ticket stores zero -- while a seeded generator decides whose turn it is, which
// stands for any timing of the waves.  Checked: every unit is taken exactly once, every queue
// hands out units + workers tickets, every counter is zero afterwards.
extern "C" perq_status_t perq_schedule_selftest(int64_t n_units, int32_t n_blocks, int32_t workers_per_block,
                                                uint64_t seed, int32_t launches) {
    namespace sch = perq::schedule;
    if (n_units <= 0 || n_blocks <= 0 || workers_per_block <= 0 || launches <= 0) return PERQ_ERR_INVALID_ARG;
    if (n_units >= ((int64_t)1 << 31) || (int64_t)n_blocks * workers_per_block >= ((int64_t)1 << 24))
        return PERQ_ERR_INVALID_ARG;
    const uint32_t W = (uint32_t)n_blocks * (uint32_t)workers_per_block, U = (uint32_t)n_units;
    if (!sch::queues_usable(n_blocks, W, n_units)) return PERQ_ERR_UNSUPPORTED;
    std::vector<uint32_t> ctr(sch::kQueues, 0u);            // one set, kept across the launches
    struct Worker {
        uint32_t queue, cur, nxt, nw;
        uint32_t pending;      // ticket drawn and not yet read
        bool has_pending, drawing;
    };
    uint64_t rng = seed * 0x9E3779B97F4A7C15ull + 0x632BE59BD9B4E019ull;
    auto next_rand = [&]() {
        rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
        return rng;
    };
    for (int32_t launch = 0; launch < launches; ++launch) {
        std::vector<uint32_t> taken(U, 0u), tickets(sch::kQueues, 0u);
        std::vector<Worker> wk(W);
        std::vector<uint32_t> active(W);
        for (uint32_t w = 0; w < W; ++w) {
            const uint32_t block = w / (uint32_t)workers_per_block;
            wk[w] = Worker{sch::queue_of_block(block), w, w + W, U, 0u, false, true};
            active[w] = w;
        }
        auto draw = [&](Worker& k) {
            k.pending = ctr[k.queue]++;
            ++tickets[k.queue];
            k.has_pending = true;
        };
        auto fetch = [&](Worker& k) -> uint32_t {
            if (!k.drawing) return U;
            if (!k.has_pending) return U + 1u;                  // (a read without a draw: flagged below)
            k.has_pending = false;
            const sch::QueuePlan qp = sch::queue_plan(U, W, k.queue);
            if (k.pending == qp.last_ticket) ctr[k.queue] = 0u;
            if (k.pending < qp.units) return sch::unit_of_ticket(qp, k.pending);
            k.drawing = false;
            return U;
        };
        std::vector<bool> started(W, false);
        while (!active.empty()) {
            const size_t pick = (size_t)(next_rand() % active.size());
            const uint32_t w = active[pick];
            Worker& k = wk[w];
            if (!started[w]) {
                // start of the kernel: the first two units are requested, one ticket drawn and read
                started[w] = true;
                draw(k);
                k.nw = fetch(k);
                if (k.nw > U) return PERQ_ERR_INTERNAL;
                continue;
            }
            // one pass of the kernel's loop body: the unit is processed, the next ticket drawn at the
            // refill of the buffer and read at the end
            if (k.cur >= U) return PERQ_ERR_INTERNAL;
            ++taken[k.cur];
            if (k.drawing) draw(k);
            k.cur = k.nxt;
            k.nxt = k.nw;
            k.nw = fetch(k);
            if (k.nw > U) return PERQ_ERR_INTERNAL;
            if (k.cur >= U) {
                if (k.has_pending) return PERQ_ERR_INTERNAL;
                active[pick] = active.back();
                active.pop_back();
            }
        }
        for (uint32_t u = 0; u < U; ++u)
            if (taken[u] != 1u) return PERQ_ERR_INTERNAL;
        for (uint32_t q = 0; q < sch::kQueues; ++q) {
            const sch::QueuePlan qp = sch::queue_plan(U, W, q);
            if (tickets[q] != qp.units + W / sch::kQueues || ctr[q] != 0u) return PERQ_ERR_INTERNAL;
        }
    }
    return PERQ_OK;
}
