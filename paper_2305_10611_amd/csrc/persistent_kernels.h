// Launch interface of the persistent (one launch for all depth levels) kernels and of the probe that
// measures what synchronising workgroups inside a kernel costs on this part.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "cell_kernels.h"

namespace acrobat {

constexpr int kLstmSlots = 16;           // sequences per node block of the LSTM launch
constexpr int kLstmMaxBlocks = 16;       // its node blocks at most (two per XCD; at H = 512 two workgroups per compute unit)
constexpr int kPersistMaxBlocks = 8;     // groups of the probe at most (one per XCD)
constexpr int kPersistMaxColBlocks = 32;   // workgroups per node block at most (H = 512)
constexpr int kPersistCounterStride = 32;  // uint32 between two groups' arrival counters of the probe (one cache line each)
// synchronisation words of one context: the probe's flag lines [group][consumer][producer], arrival counters, status
constexpr int kPersistFlagWords = kPersistMaxBlocks * kPersistMaxColBlocks * kPersistMaxColBlocks;
constexpr int kPersistSyncWords = kPersistFlagWords + kPersistMaxBlocks * kPersistCounterStride + 1;

// The LSTM recurrence of a whole mini-batch in one launch.  The sequences are dealt out to node blocks of 16
// slots; workgroup (block nb, column block cb) keeps the 64 rows of W_h that belong to hidden units
// 16 cb .. 16 cb + 15 (all four gates) in registers for every step and owns those units of the block's
// sequences.  After step t the workgroups of a block exchange h_t through the arena and arrive at the block's
// counter; blocks never wait for each other.
struct LstmPersistentArgs {
  int32_t n_blocks;          // node blocks in use, 1 .. kLstmMaxBlocks
  int32_t H;                 // hidden size (the kernel is instantiated for 128, 256 and 512)
  const int32_t* slot_row0;  // [n_blocks * 16] first arena row of the slot's sequence
  const int32_t* slot_len;   // [n_blocks * 16] its length, non-increasing inside a block, 0 = empty slot
  const float* Wh;           // [4H, H], gate order (i, f, o, u)
  const float* xp;           // [rows, 4H] hoisted input transform (bias included)
  float* h; float* c;        // arena [rows, H], row = slot_row0 + t
  uint32_t h_bytes;          // size of h in bytes (< 2^32: the exchanged rows are read through a buffer resource)
  unsigned* counters;        // [n_blocks * kPersistCounterStride]: arrivals of a block's workgroups, and behind each the
                             // workgroups that have left; zero at launch, and zero again when the launch has completed
  unsigned* status;          // set to 1 by a workgroup whose wait ran out (the kernel then drains and ends)
  int32_t max_polls;         // bound of every wait, in polls of the counter
};

// True if lstm_persistent can run this shape (H instantiated, blocks fit one launch, every workgroup resident
// at once on the current device).  *why (may be null) names the reason when it cannot.
bool lstm_persistent_eligible(int32_t H, int32_t n_blocks, const char** why);
hipError_t launch_lstm_persistent(const LstmPersistentArgs& a, hipStream_t stream, const LaunchEvents& ev = LaunchEvents());

// The two recurrences of a bidirectional RNN (single gate: h_t = sigmoid(W_h h_prev + xp_t)) in one launch.
// Sequences are dealt to blocks of 16 slots; block 2 i + dir runs direction dir (0 forward, 1 backward) of the
// i-th group of sequences.  Workgroup (block, column block cb) keeps the 16 rows of that direction's W_h that
// belong to hidden units 16 cb .. 16 cb + 15 in registers (wavefront w: columns w H/4 .. of those rows, a quarter
// of the contraction) and exchanges h with the other H / 16 workgroups of its block after every step, exactly as
// the LSTM kernel does.
constexpr int kRnnSlots = 16;
constexpr int kRnnMaxBlocks = 32;
struct RnnPersistentArgs {
  int32_t n_blocks;          // blocks in use (even), 2 .. kRnnMaxBlocks
  int32_t H;                 // hidden size (instantiated for 128, 256 and 512)
  const int32_t* slot_row0;  // [n_blocks / 2 * 16] first row of the slot's sequence (both directions use the same slots)
  const int32_t* slot_len;   // [n_blocks / 2 * 16] its length, non-increasing inside a block, 0 = empty slot
  const float* Wh[2];        // [H, H] per direction
  const float* xp[2];        // [rows, H] hoisted input transform (bias included)
  const float* h_init[2];    // [H] state before the first step
  float* h[2];               // [rows, H]; forward step t of a sequence writes row row0 + t, backward row0 + len - 1 - t
  uint32_t h_bytes;          // size of one h array in bytes (< 2^32)
  unsigned* counters;        // [kRnnMaxBlocks * kPersistCounterStride], zero at launch and again when the launch has completed
  unsigned* status;
  int32_t max_polls;
};
bool rnn_persistent_eligible(int32_t H, int32_t n_blocks, const char** why);
hipError_t launch_rnn_persistent(const RnnPersistentArgs& a, hipStream_t stream, const LaunchEvents& ev = LaunchEvents());

// Fills n uint32 with a value (a kernel, so that a captured graph holds no memset node).
hipError_t launch_fill_u32(unsigned* p, unsigned value, int n, hipStream_t stream);

// ---- probe: cost of a barrier among workgroups inside one kernel -------------------------------------
// `groups` x `group_size` workgroups; each round every workgroup stores `store_floats` floats of its own,
// arrives at its group's counter, waits until the whole group has arrived, and reads `load_floats` floats
// that the group stored.  Workgroup b belongs to group b % groups (same_xcd: the members of a group then
// share an XCD when groups == 8) or b / group_size (members spread over all XCDs).
struct SyncProbeArgs {
  int32_t groups, group_size, rounds;
  int32_t same_xcd;       // 1: group = workgroup id % groups, 0: group = workgroup id / group_size
  int32_t style;          // 0: counter + release / acquire fences, 1: counter without fences, 2: flag lines without fences,
                          // 3: style 1 with payload addresses of its own for every round and plain payload loads
  int32_t write_through;  // style 0 only: 1 = payload stores are agent-scope atomic stores (write through), 0 = plain stores
  int32_t store_floats, load_floats;  // payload per workgroup and round (multiples of 256, <= 16384)
  float* payload;         // [groups * group_size * store_floats * 2] (two generations; style 3: * rounds, one per round)
  unsigned* counters;     // [groups * kPersistCounterStride], zero at launch
  unsigned* flags;        // [kPersistFlagWords], zero at launch
  unsigned* status;
  int32_t max_polls;
  // per workgroup: ticks of the 100 MHz clock summed over the rounds, spent in
  // [0] payload stores + workgroup barrier, [1] release + arrival, [2] polling, [3] acquire + workgroup barrier,
  // [4] payload loads
  unsigned long long* ticks;  // [groups * group_size * 5]
  unsigned* stale;            // [1] zero at launch: payload elements read that did not hold the round's value
};
hipError_t launch_sync_probe(const SyncProbeArgs& a, hipStream_t stream, const LaunchEvents& ev = LaunchEvents());

}  // namespace acrobat
