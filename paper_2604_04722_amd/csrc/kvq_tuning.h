// Process-wide launch-shape overrides (tests and tuning runs; normal use never touches them).
//
// The hot-path entry points read these plain ints and nothing else: the environment is looked at ONCE, when the table
// is first needed, and never again.  kvq_tuning_set() changes an entry afterwards (the tests use it to force a code
// path); it is not synchronised with calls running on other threads.
#pragma once

namespace kvq {

struct Tuning {
    int attn_splits;            // 0: automatic; 1..64: workgroups a (sequence, head) is split over
    int attn_waves;             // 0: automatic; 1, 2, 3, 4, 8: waves per attention workgroup
    int attn_longest_first;     // -1: automatic; 0 / 1: longest-first launch order off / on
    int attn_by_class;          // whole waves per class when a wave has at most this many units on average (0: never)
    int append_bulk_min_T;      // smallest T that takes the lane-per-token append kernels
    int append_stream_min;      // tokens of one class in a 64-token tile from which that class is stored non-temporally
    int append_block_min_T;     // smallest T that takes the block-at-a-time prefill writer
    int controller_no_mfma;     // 1: bulk controller on the vector ALU even for widths 32/64/128
    int controller_waves;       // 0: automatic; 4 or 8 waves per workgroup of the MFMA controller launch
    int controller_wg_per_cu;   // 0: automatic; 1..4 workgroups per compute unit of the MFMA controller launch
    int train_no_mfma;          // 1: training step's middle layer on the vector ALU
};

Tuning &tuning();               // defined once in kvq_cache.hip

}  // namespace kvq
