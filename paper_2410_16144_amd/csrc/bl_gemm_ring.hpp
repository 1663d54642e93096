// Ring depths and wait counts of the prefill kernel's operand pipeline (bl_gemm.hip), as compile-time constants in a
// header of their own: the kernel takes them from here, and so does the host-side model that replays the kernel's
// issue order and checks every wait (tests/ring_model).  Plain C++, no device code.
//
// The pipeline, per thread and K step i (one packed tile per K group):
//   - activations: the tile of step i + kLead is requested (global -> LDS, kRQ loads per thread of a loader wave, written
//     as assembly, so the compiler neither sees, drops nor moves them) into stage (i + kLead) % kStages;
//   - weights: the packed tiles of step i + kWR - 1 are loaded into registers (NT ordinary loads: the compiler sees
//     them and may DROP the ones whose values are never used, which is what happens in the loop's unrolled tail);
//   - the barrier that ends step i publishes the activation tile of step i + 2 (step i + 1 reads its first half during
//     its predecessor's second half).  Vector memory operations complete in issue order and one counter (vmcnt)
//     counts all of them, so "tile i + 2 has landed" is "at most n operations are outstanding", n = the operations
//     this thread has issued since that tile's request.
#pragma once

namespace bl {

template <int MB, int H, int WK, int WN>
struct GemmRing {
    static constexpr int kNT = (H + 1) / 2;            // packed 64-row tiles a wave loads per step
    static constexpr int kStages = WK == 1 ? 8 : 6;    // LDS stages of the activation ring
    // a stage is WK tiles of 32 MB token rows = WK * 2 MB slabs of 1 KiB, one wave-load each, dealt to the WN * WK waves:
    // a loader wave issues kRQ of them per step (the other waves none)
    static constexpr int kRQ = (WK * 2 * MB + WN * WK - 1) / (WN * WK);
    static constexpr int kLead = 4;                    // the tile of step i + kLead is requested during step i
    static constexpr int kWR = kNT == 1 ? 8 : 4;       // register ring of packed weight tiles, steps i .. i + kWR - 1
    static constexpr int kUnroll = 8;                  // steps per trip of the main loop; the rest is the tail
    // Main loop: since the request of tile i + 2 (first thing in step i + 2 - kLead) the thread has issued that step's
    // weight loads and kLead - 2 whole steps: (kLead - 2) * (kRQ + kNT) + kNT operations.  The count below leaves the
    // kNT out, i.e. it also waits for the weight tiles of the requesting step: stricter than needed, never weaker.
    static constexpr int kYounger = (kLead - 2) * (kRQ + kNT);
    // Tail (the steps after the last whole trip): their weight loads feed nothing and the compiler removes them, so only
    // the requests are sure to have been issued: kLead - 2 steps of kRQ each.
    static constexpr int kYoungerTail = (kLead - 2) * kRQ;
    // Prologue: kWR - 1 steps of weight loads, then the requests of tiles 0 .. kLead - 1 back to back.  The wait leaves
    // only the requests of tiles 3 .. kLead - 1 outstanding, so tiles 0, 1 AND 2 have landed: the barrier that ends step 0
    // is meant to publish tile 2, but only kRQ + kNT + kRQ operations follow its request by then, fewer than kYounger.
    static constexpr int kPrologueWait = (kLead - 3) * kRQ;

    static_assert(kLead >= 3, "the prologue waits for all but the last requested tiles");
    static_assert(kStages >= kLead + 1, "a stage is rewritten only after the barrier that ended its last read");
    static_assert(kYounger < 16 && kYoungerTail < 16 && kPrologueWait < 16, "fits the low vmcnt field");
    static_assert(kUnroll % kWR == 0, "register ring slots are compile-time phases of the unrolled loop");
};

// The matrix-core decode kernel's one-off copy of the quantized activations into LDS (bl_gemv.hip, QMODE 1): the copy's
// global -> LDS loads are issued first, then one batch of U weight tiles; the wait that precedes the barrier allows
// exactly those U loads to be outstanding.
template <int U>
struct LdsCopyWait {
    static constexpr int kYounger = U;
    static_assert(U >= 0 && U < 16, "fits the low vmcnt field");
};

}  // namespace bl
