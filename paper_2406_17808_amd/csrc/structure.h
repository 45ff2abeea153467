// Host-side mirror of the score-independent part of the cache state.
//
// In Alg. 2 only the CONTENT of a slot depends on the attention scores (token selection
// replaces the newest item in place).  How full every sub-cache is, where its ring head
// sits (Section 3.1 "Circular Buffers") and when it accepts are functions of the number of
// tokens seen alone, identical for every sequence and KV head.  The host therefore tracks
// them itself and never has to read anything back from the device to size a launch.
#pragma once

#include <stdint.h>

#include <string>

#include "internal.h"

namespace ckv {

// Validation of a configuration (CASCADE_OK or an error code with the reason in `why`) and the
// geometry derived from a valid one.
int check_config(const cascade_config* c, std::string& why);
void make_geom(const cascade_config* c, Geom& g);

// Text of the last failure of a call that has no context to keep it in (per host thread).
void set_init_error(const std::string& msg);
const char* init_error();

struct HostState {
    int sink_fill = 0;
    int count[kMaxCascades] = {0};
    int xi[kMaxCascades] = {0};        // ring index of the oldest item; 0 while the cascade is filling
    int64_t t = 0;                     // tokens offered to the first cascade so far
    int64_t n_seen = 0;                // tokens consumed so far
    int64_t accepted[kMaxCascades] = {0};
    int64_t discards[kMaxCascades] = {0};

    int n_cached(const Geom& g) const
    {
        int n = sink_fill;
        for (int c = 0; c < g.N; ++c) n += count[c];
        return n;
    }
};

// Structure of inserting Q tokens in order (Alg. 2 applied Q times); advances `st`.
void plan_update(const Geom& g, HostState& st, int Q, UpdatePlan& plan);

// Runs of physical rows that share one query rotation, for the state BEFORE a chunk of Q tokens.
// with_chunk: append the segment of the chunk's own keys.
void build_segments(const Geom& g, const HostState& st, bool with_chunk, int Q, SegList& out);

// Where the 64-row tiles of the packed K / V copies sit when every ring is full.  build_segments
// lists a full ring as [0, o), [o, xi), [xi, cap) with o = xi mod 64, so ring rows o + 64k ..
// o + 64k + 63 always form tile (o > 0) + k of the ring whatever xi is: as long as no o changes,
// a tile keeps its place and its content from chunk to chunk until one of its rows is written.
struct PackedLayout {
    bool full;                    // sinks and every ring are full
    int off[kMaxCascades];        // o of every ring
    int tile0[kMaxCascades];      // first tile of every ring
    int cache_tiles;              // tiles of all cached rows; the chunk's tiles follow
};
void packed_layout(const Geom& g, const HostState& st, PackedLayout& out);
bool same_offsets(const Geom& g, const PackedLayout& a, const PackedLayout& b);

// The physical slots an update may write (ring positions opened, and the resident item the
// first offers compete with), as runs [lo, hi) of slots inside one ring or the sinks; returns the
// number of runs (<= 2 per cascade + 1 for the sinks).
int touched_slot_runs(const Geom& g, const UpdatePlan& pl, int* lo, int* hi);

// The same as runs of tiles of `layout`, appended to `runs`; false if `runs` cannot hold them.
bool add_touched_tiles(const Geom& g, const PackedLayout& layout, const UpdatePlan& pl, TileRuns& runs);
bool add_tile_run(TileRuns& runs, int first, int count);

// physical slot of the r-th entry in cache order (r < n_cached)
int slot_of_rank(const Geom& g, const HostState& st, int r);

}  // namespace ckv
