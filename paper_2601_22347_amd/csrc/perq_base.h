// Base matrices of the non-power-of-two Hadamard rotation (Appendix A.1), host side.
#pragma once
#include <cstdint>

namespace perq {

// 0: m is not 4t with t odd and above 1, or no construction is known to the library for it;
// 1: Paley's first construction
// (m - 1 a prime, 3 mod 4); 2: his second (m/2 - 1 a prime, 1 mod 4).  The first is preferred.
int hadamard_base_kind(int32_t m);
// Entry (r, c), +1 or -1, of the m x m base matrix of the given kind.
int hadamard_base_entry(int32_t m, int kind, int32_t r, int32_t c);

}  // namespace perq
