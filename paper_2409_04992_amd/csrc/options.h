// Implementation switches of the library (host side only): values that force one of
// the host's choices for experiments and tests.  They live in process-wide atomics,
// are set through instattn_set_option, and start from the environment variable of the
// same name, read once per process.  An entry point takes ONE snapshot when it is
// called and decides everything from that snapshot.
#pragma once

namespace instattn {

enum Option {
    kOptChunk = 0,            // INSTATTN_CHUNK: positions per unit of the dense split pass (> 0 forces it)
    kOptRotate,               // INSTATTN_ROTATE: 1 = every unit starts its walk at a tile of its own
    kOptSparfDistributed,     // INSTATTN_SPARF_DISTRIBUTED: 1 / 0 = selection spread over stretches, or never
    kOptSparfThreeLaunches,   // INSTATTN_SPARF_THREE_LAUNCHES: 1 = never the one-launch kernel
    kOptSparfWide,            // INSTATTN_SPARF_WIDE: 1 / 0 = the one-launch kernel's wide forms always, or never
    kOptSparfSplitTail,       // INSTATTN_SPARF_SPLIT_TAIL: 1 = selection and gather never share a launch
    kOptCompact,              // INSTATTN_COMPACT: 1 / 0 = dense split pass over the compacted unit list always, or never
    kOptMhaRing,              // INSTATTN_MHA_RING: 1 / 0 = vector-ALU split pass through its LDS ring always, or never
    kNumOptions
};

// A negative value means "not set": the host decides.
struct Options {
    int v[kNumOptions];
    int operator[](Option o) const { return v[o]; }
};

Options options_snapshot();
const char* option_name(int o);

}  // namespace instattn
