// Work plan shared by the EGAE scan and the loss kernels.
//
// The response-packed token array is cut into tiles of at most kTileTokens
// tokens that never straddle two sequences, at multiples of kTileTokens of the
// packed index: a sequence is a short first tile up to the next multiple, full
// tiles that are aligned blocks of the arrays, and a short last tile.  A tile is described by 16 bytes,
// so a wavefront learns everything about its tokens (which sequence, how far
// into it, how many tiles follow) from ONE load instead of a chain of dependent
// look-ups in the offset arrays.
//
// Order of the list.  The scan's only dependency runs from a tile to the tiles
// AFTER it in the same sequence, and a kernel that takes one tile per workgroup
// starts them in list order.  So the list is sorted by `after` ("level"): first
// every sequence's last tile, then every second-to-last one, ...  A tile's
// dependencies then started (number of sequences at least that long) workgroups
// earlier -- thousands on the long-CoT batches of Sec. 4 -- and have published
// long before it looks for them; with the sequences simply laid end to end they
// would start together with it and every tile would sit out a round trip through
// memory.  Levels kLevels and up (sequences beyond 32 K tokens) follow the sorted
// part, each sequence's tiles together, innermost level first.
//
// A plan is one block of device memory:
//   header (256 B)   tile count, the sizes it was built for, the sizes of the
//                    policy / value token sets of Sec. 3.2
//   tiles[cap]       the descriptors
//   frames[cap]      per aligned block ("frame") of kTileTokens tokens of the arrays:
//                    which sequence its first token belongs to, where that sequence
//                    and its policy tokens (a prefix, Sec. 3.2) end and whether it is
//                    finished.  The loss kernels, which have no dependency between
//                    tokens, walk frames instead of tiles: every access is a whole,
//                    aligned one, and a frame inside one sequence (most are) needs
//                    no look-up in the offset arrays
//   scan_words[cap][8]   what a tile of the scan publishes for the tiles to its
//                    left, {tag << 32 | float bits} each: A hi, A lo, R hi, R lo
//                    of the tile alone, then the same four with everything to
//                    its right included.  Indexed by Tile::slot(), which numbers
//                    a sequence's tiles consecutively.
//   finish_words[kFinishGroups][kFinishWords]   partial sums of a reduction
//                    kernel's workgroups, in the same tagged form
// Whoever builds the list (tppo_select, tppo_plan_build, or an entry point that
// was given no plan and builds its own in its workspace) zeroes all tagged
// words.  Every later launch tags what it writes with its own call number
// (never 0, never repeated inside a process), so words left by earlier calls
// on the same plan never look ready and a plan needs no clearing between calls.
#pragma once
#include "common.h"

namespace tppo {

constexpr int kTileTokens = 1024;
constexpr int kTileShift = 11;                 // pos_len keeps (tokens - 1) in the low bits
constexpr int kLevels = 32;                    // levels the list is sorted by
constexpr int kScanWords = 8;                  // tagged words per tile
constexpr int kBuildThreads = 1024;
constexpr int kFinishGroups = 2048;            // most workgroups a reduction kernel may launch
constexpr int kFinishWords = 10;               // tagged words per workgroup: five sums as hi + lo

static_assert(kTileTokens <= (1 << kTileShift), "Tile::pos_len packs the length below the tile number");

struct Tile {
    int32_t start;     // response-packed index of the tile's first token
    int32_t pos_len;   // (tile number inside the sequence << 11) | (tokens in the tile - 1)
    int32_t seg;       // sequence the tile belongs to
    int32_t after;     // tiles after it in the same sequence (0: it holds the sequence's last token)
    __device__ __forceinline__ int len() const { return (pos_len & ((1 << kTileShift) - 1)) + 1; }
    __device__ __forceinline__ int number() const { return pos_len >> kTileShift; }
    // a tile lies inside one aligned block of kTileTokens tokens of the arrays: the block's first token, and
    // where in the block the tile begins (0 for every tile but a sequence's first)
    __device__ __forceinline__ int base() const { return start & ~(kTileTokens - 1); }
    __device__ __forceinline__ int begin() const { return start & (kTileTokens - 1); }
    // consecutive for the tiles of a sequence, unique in the batch, below plan_max_tiles(n_resp, B)
    __device__ __forceinline__ int slot() const { return start / kTileTokens + seg; }
};

struct PlanHeader {
    int32_t n_tiles;               // tiles in the list
    int32_t B, n_resp;             // what the plan was built for; a consumer called with other sizes refuses it
    int32_t has_sets;              // n_policy / n_value are valid (the builder knew keep_len)
    long long n_policy, n_value;   // tokens in the policy set / the value set (Sec. 3.2)
    int32_t cap;                   // descriptors the plan has room for (fixes where the tagged words start)
};

// What is known about frame f (tokens f * kTileTokens ...) without looking at the offset arrays: the sequence
// that holds its first token and, when that one ends inside the frame, the sequence that follows it there.
// Tokens of the frame at or beyond `end2` (a third sequence: only after one of fewer than kTileTokens
// tokens) are looked up in the offset arrays.
struct FrameDesc {
    int32_t seg;       // sequence of the frame's first token
    int32_t end;       // response-packed index one past that sequence's last token
    int32_t pol_end;   // one past its last policy token (Sec. 3.2: the first keep_len tokens of the window)
    int32_t fin;       // != 0: the sequence is finished, its tokens are value tokens
    int32_t seg2;      // the sequence of token `end` (seg, with end2 == end, when the builder did not look)
    int32_t end2, pol_end2, fin2;
};
static_assert(sizeof(FrameDesc) == 32, "a frame's descriptor is one 32-byte scalar load");

struct Plan {
    PlanHeader* hdr;
    Tile* tiles;
    FrameDesc* frames;                   // [cap], by frame number; the set fields are meaningful when hdr->has_sets
    unsigned long long* scan_words;      // [cap][kScanWords], by Tile::slot()
    unsigned long long* finish_words;    // [kFinishGroups][kFinishWords]
    int cap;
};

// most tiles a batch can have: a sequence has one more tile than multiples of kTileTokens inside it
static constexpr int64_t plan_max_tiles(int64_t n_resp, int64_t B) { return n_resp / kTileTokens + B + 1; }

static constexpr size_t plan_bytes_for(int64_t cap) {
    return 256 + round_up((size_t)cap * sizeof(Tile), 256) + round_up((size_t)cap * sizeof(FrameDesc), 256) +
           round_up((size_t)cap * kScanWords * 8, 256) +
           (size_t)kFinishGroups * kFinishWords * sizeof(unsigned long long);
}

__host__ __device__ __forceinline__ Plan plan_view(void* raw, int64_t cap) {
    char* p = static_cast<char*>(raw);
    Plan pl;
    pl.hdr = reinterpret_cast<PlanHeader*>(p);
    p += 256;
    pl.tiles = reinterpret_cast<Tile*>(p);
    p += ((size_t)cap * sizeof(Tile) + 255) / 256 * 256;
    pl.frames = reinterpret_cast<FrameDesc*>(p);
    p += ((size_t)cap * sizeof(FrameDesc) + 255) / 256 * 256;
    pl.scan_words = reinterpret_cast<unsigned long long*>(p);
    p += ((size_t)cap * kScanWords * 8 + 255) / 256 * 256;
    pl.finish_words = reinterpret_cast<unsigned long long*>(p);
    pl.cap = (int)cap;
    return pl;
}

// a consumer's view: the capacity the builder used is in the header
__device__ __forceinline__ Plan plan_open(void* raw) {
    return plan_view(raw, load_uniform(&static_cast<const PlanHeader*>(raw)->cap));
}

// a wave-uniform descriptor, through the scalar data cache
__device__ __forceinline__ Tile load_tile(const Tile* p) {
    typedef int int4v __attribute__((ext_vector_type(4)));
    const int4v x = *(const int4v __attribute__((address_space(4)))*)(p);
    return Tile{x[0], x[1], x[2], x[3]};
}

__device__ __forceinline__ FrameDesc load_frame(const FrameDesc* p) {
    typedef int int8v __attribute__((ext_vector_type(8)));
    const int8v x = *(const int8v __attribute__((address_space(4)))*)(p);
    return FrameDesc{x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7]};
}

// A zero the compiler cannot see through.  Added to a wave-uniform address it keeps the load a VECTOR load: with
// thousands of wavefronts each fetching a line of its own, loads through the scalar data cache were measured
// at 4000-6000 cycles, against about 1200 for vector loads issued at the same moment.
__device__ __forceinline__ int opaque_zero() {
    int z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// a descriptor as a vector load (every lane the same 16 bytes) ...
typedef int tile_bits __attribute__((ext_vector_type(4)));
__device__ __forceinline__ tile_bits fetch_tile(const Tile* p, int zero) {
    return *reinterpret_cast<const tile_bits*>(reinterpret_cast<const char*>(p) + zero);
}
// ... and back in scalar registers, where lengths and branches on it cost nothing
__device__ __forceinline__ Tile uniform_tile(tile_bits x) {
    return Tile{__builtin_amdgcn_readfirstlane(x[0]), __builtin_amdgcn_readfirstlane(x[1]),
                __builtin_amdgcn_readfirstlane(x[2]), __builtin_amdgcn_readfirstlane(x[3])};
}

// A consumer trusts no descriptor it has not checked: a plan is caller-held memory, and a descriptor decides
// which addresses are touched.  True when every token, side load and tagged word the tile names exists.
__device__ __forceinline__ bool tile_valid(const Tile& t, int n_resp, int B, int cap) {
    const int len = t.len();
    return t.start >= 0 && t.start <= n_resp - len && t.seg >= 0 && t.seg < B && t.after >= 0 && t.number() >= 0 &&
           t.after < cap - t.slot() && t.begin() + len <= kTileTokens &&
           (t.after == 0 || (t.begin() + len == kTileTokens && t.start + len < n_resp));
}

// number of 8-byte tagged words of a plan (scan words, then finish words: contiguous but for padding)
__host__ __device__ static inline int64_t plan_words(int64_t cap) {
    return (int64_t)(((size_t)cap * kScanWords * 8 + 255) / 256 * 256) / 8 + (int64_t)kFinishGroups * kFinishWords;
}

// One workgroup per 1024 sequences builds the list (measured on 8704 sequences: the descriptor stores, one
// cache line per lane, are what takes the time, which is why large batches spread them over several).
constexpr int kBuildSeqsPerPart = 1024, kBuildMaxParts = 16;
static inline int build_parts(int64_t B) {
    const int64_t n = (B + kBuildSeqsPerPart - 1) / kBuildSeqsPerPart;
    return n < 1 ? 1 : n > kBuildMaxParts ? kBuildMaxParts : (int)n;
}

__device__ __forceinline__ int tiles_of(int len) { return (len + kTileTokens - 1) / kTileTokens; }

// the descriptors of one sequence: tokens [lo, lo + len) of the response-packed domain, list positions
// first .. first + tiles_of(len) - 1
__device__ __forceinline__ void emit_tiles(Tile* __restrict__ tiles, int cap, int first, int seg, int lo, int len) {
    const int cnt = tiles_of(len);
    for (int c = 0; c < cnt; ++c) {
        Tile d;
        d.start = lo + c * kTileTokens;
        d.pos_len = (c << kTileShift) | (min(kTileTokens, len - c * kTileTokens) - 1);
        d.seg = seg;
        d.after = cnt - 1 - c;
        if (first + c < cap) tiles[first + c] = d;             // overlapping sequences cannot overflow the list
    }
}

// a tagged word: {tag, float}.  A double travels as two of them (hi + lo).
__device__ __forceinline__ unsigned long long pack_word(uint32_t tag, float v) {
    return ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
}

__device__ __forceinline__ void publish(unsigned long long* p, uint32_t tag, double x) {
    const float hi = (float)x, lo = (float)(x - (double)hi);
    __hip_atomic_store(p, pack_word(tag, hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, pack_word(tag, lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One poll of a published double; true when both halves carry this call's tag.
__device__ __forceinline__ bool poll(const unsigned long long* p, uint32_t tag, double& x) {
    const unsigned long long w0 = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long w1 = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    x = (double)__uint_as_float((unsigned)w0) + (double)__uint_as_float((unsigned)w1);
    return (uint32_t)(w0 >> 32) == tag && (uint32_t)(w1 >> 32) == tag;
}

// The next call number (host side; never 0).
uint32_t next_call_tag();

// Enqueue the kernel that builds a plan for (resp_off, done[, keep_len]) in `plan_raw` (plan_bytes_for(cap)
// bytes) and zeroes its tagged words.  keep_len may be NULL (no set sizes).  n_resp < 0: the kernel takes
// resp_off[B] for it (a caller whose offsets are still being computed on the stream).
int launch_plan_build(const int32_t* resp_off, const int32_t* keep_len, const int32_t* done, int64_t B,
                      int64_t n_resp, int64_t cap, void* plan_raw, int32_t* status, hipStream_t s);

}  // namespace tppo
