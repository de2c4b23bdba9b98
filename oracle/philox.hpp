// TEST INFRASTRUCTURE ONLY.  This directory is the CPU oracle: a plain, slow,
// scalar definition of what the sharded random-number path must compute.
// Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
// it.  It shares no code with the HIP library and neither includes the other.
//
// Philox4x32-10, the counter-based generator of Salmon, Moraes, Dror and Shaw
// ("Parallel random numbers: as easy as 1, 2, 3", SC'11).  It stands in for the
// "local random value generator lambda" of the paper's Algorithm 1 (Section 5),
// which the paper leaves to a vendor library.
#pragma once
#include <cstdint>

namespace oracle {

struct Block {
  uint32_t w[4];
};

// Ten rounds of the Philox-4x32 bijection on a 128-bit counter and a 64-bit key.
Block philox4x32_10(const uint32_t ctr[4], const uint32_t key[2]);

// Where an element's draw lives: a 128-bit counter and the output word to take.
// Two layouts (Algorithm 1, "virtualize thread index and offset"):
//  * theta == 0, this build's default reading: one flat stream, position
//    p = offset + j, counter (lo32 b, hi32 b, 0, 0) with b = p / 4, word p % 4.
//  * theta > 0, Algorithm 1 to the letter with a global thread count theta: virtual
//    thread tau = j mod theta, virtual offset beta = offset + j / theta; the
//    generator is called with (seed, tau, beta): counter (lo32 q, hi32 q, lo32 tau,
//    hi32 tau) with q = beta / 4, word beta % 4.
struct Slot {
  uint32_t ctr[4];
  uint32_t word;
};
Slot slot_of(uint64_t offset, uint64_t j, uint64_t theta);

// The draw at stream position `p` under `seed`: key = (lo32 seed, hi32 seed),
// counter = (lo32 b, hi32 b, 0, 0) with b = p / 4, and the word picked is p % 4.
// One full generator call per draw: the oracle never reuses a block.
uint32_t draw(uint64_t seed, uint64_t p);

// Word `word` (0..3) of the block at the slot's counter.
uint32_t draw_word(uint64_t seed, const Slot& slot, uint32_t word);

}  // namespace oracle
