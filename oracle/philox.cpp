// TEST INFRASTRUCTURE ONLY (see philox.hpp).
#include "philox.hpp"

namespace oracle {

namespace {
// Constants of the published Philox-4x32 definition.
constexpr uint32_t kMul0 = 0xD2511F53u;   // multiplies counter word 0
constexpr uint32_t kMul1 = 0xCD9E8D57u;   // multiplies counter word 2
constexpr uint32_t kWeyl0 = 0x9E3779B9u;  // key word 0 bump (golden ratio)
constexpr uint32_t kWeyl1 = 0xBB67AE85u;  // key word 1 bump (sqrt(3) - 1)
}  // namespace

Block philox4x32_10(const uint32_t ctr[4], const uint32_t key[2]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {  // the key is bumped before every round but the first
      k0 += kWeyl0;
      k1 += kWeyl1;
    }
    const uint64_t prod0 = static_cast<uint64_t>(kMul0) * c0;
    const uint64_t prod1 = static_cast<uint64_t>(kMul1) * c2;
    const uint32_t hi0 = static_cast<uint32_t>(prod0 >> 32);
    const uint32_t lo0 = static_cast<uint32_t>(prod0);
    const uint32_t hi1 = static_cast<uint32_t>(prod1 >> 32);
    const uint32_t lo1 = static_cast<uint32_t>(prod1);
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0;
    c1 = n1;
    c2 = n2;
    c3 = n3;
  }
  return Block{{c0, c1, c2, c3}};
}

uint32_t draw(uint64_t seed, uint64_t p) {
  const uint64_t b = p / 4;
  const uint32_t ctr[4] = {static_cast<uint32_t>(b), static_cast<uint32_t>(b >> 32), 0u, 0u};
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  return philox4x32_10(ctr, key).w[p % 4];
}

Slot slot_of(uint64_t offset, uint64_t j, uint64_t theta) {
  Slot s;
  if (theta == 0) {
    const uint64_t p = offset + j;
    const uint64_t b = p / 4;
    s.ctr[0] = static_cast<uint32_t>(b);
    s.ctr[1] = static_cast<uint32_t>(b >> 32);
    s.ctr[2] = 0;
    s.ctr[3] = 0;
    s.word = static_cast<uint32_t>(p % 4);
  } else {
    const uint64_t tau = j % theta;
    const uint64_t beta = offset + j / theta;
    const uint64_t q = beta / 4;
    s.ctr[0] = static_cast<uint32_t>(q);
    s.ctr[1] = static_cast<uint32_t>(q >> 32);
    s.ctr[2] = static_cast<uint32_t>(tau);
    s.ctr[3] = static_cast<uint32_t>(tau >> 32);
    s.word = static_cast<uint32_t>(beta % 4);
  }
  return s;
}

uint32_t draw_word(uint64_t seed, const Slot& slot, uint32_t word) {
  const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
  return philox4x32_10(slot.ctr, key).w[word];
}

}  // namespace oracle
