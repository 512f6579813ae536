// Work list shared by the EGAE scan and the loss reductions.
//
// The response-packed token array is cut into chunks of at most kChunkTokens
// tokens that never straddle two sequences.  A chunk is described by 16 bytes,
// so a workgroup learns everything about its tokens (which sequence, where the
// sequence ends, how far into the sequence it is) from ONE load instead of a
// chain of dependent look-ups in the offset arrays.  Chunks are listed in
// processing order: last sequence first and, inside a sequence, last chunk
// first -- the order in which a right-to-left scan can consume them.
#pragma once
#include "common.h"

namespace tppo {

constexpr int kChunkThreads = 256;
constexpr int kChunkTpt = 8;                                   // tokens per thread
constexpr int kChunkTokens = kChunkThreads * kChunkTpt;        // 2048
constexpr int kBuildThreads = 1024;

static_assert(kChunkTokens == 2048, "Chunk::pos_len packs the length in 11 bits");

struct Chunk {
    int32_t start;     // response-packed index of the chunk's first token
    int32_t pos_len;   // (chunk number inside the sequence << 11) | (tokens in the chunk - 1)
    int32_t seg;       // sequence the chunk belongs to
    int32_t after;     // chunks after it in the same sequence (0: it holds the sequence's last token)
    __device__ __forceinline__ int len() const { return (pos_len & (kChunkTokens - 1)) + 1; }
    __device__ __forceinline__ int number() const { return pos_len >> 11; }
};

static inline int64_t max_chunks(int64_t n_resp, int64_t B) { return n_resp / kChunkTokens + B + 1; }

// `parts` workgroups build the list together (one per 1024 sequences, see
// build_parts; measured on 8704 sequences: 3 workgroups take 20 us off the
// single-workgroup time, 9 another 2 us).  Workgroup `part` owns a contiguous range of the
// sequences (in reverse order: last sequence first) and, inside it, thread t a
// contiguous block, so there is ONE workgroup-wide prefix sum: pass A adds up
// the chunk counts of the block, the scan turns the totals into each block's
// first list position, pass B re-reads the (cache-resident) offsets and writes
// the descriptors.  Where its range starts in the list a workgroup finds out by
// itself, by adding up the chunk counts of all sequences before its range -- a
// coalesced read of offsets that sit in the cache, which is cheaper than a
// second launch.  (Measured with device timers on 8704 sequences / 24 k
// chunks: the descriptor stores, one cache line per lane, are what takes the
// time -- ~8 us per 11 k descriptors in one workgroup, which is why large
// batches spread them over several; staging the metadata through LDS or giving
// every list position its own thread with a bisection is no faster.)
// Sequences with a bad layout (negative length, out of range) contribute no
// chunk and set the status bit.  n_chunks[0] receives the total.
constexpr int kBuildSeqsPerPart = 1024, kBuildMaxParts = 16;
static inline int build_parts(int64_t B) {
    const int64_t n = (B + kBuildSeqsPerPart - 1) / kBuildSeqsPerPart;
    return n < 1 ? 1 : n > kBuildMaxParts ? kBuildMaxParts : (int)n;
}

__device__ __forceinline__ int chunks_of(const int32_t* __restrict__ resp_off, int i, int n_resp, int& lo, int& len,
                                         int32_t* status) {
    lo = resp_off[i];
    const int hi = resp_off[i + 1];
    len = 0;
    if (lo < 0 || hi < lo || hi > n_resp) {
        if (status) set_status(status, TPPO_STATUS_BAD_LAYOUT);
        return 0;
    }
    len = hi - lo;
    return (len + kChunkTokens - 1) / kChunkTokens;
}

__device__ __forceinline__ void build_chunks(const int32_t* __restrict__ resp_off, int B, int n_resp,
                                             Chunk* __restrict__ chunks, int cap,
                                             int32_t* __restrict__ n_chunks, int32_t* status, int part, int parts) {
    __shared__ int s_wave[2][kBuildThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (part == 0 && tid == 0 && (resp_off[0] != 0 || resp_off[B] != n_resp)) set_status(status, TPPO_STATUS_BAD_LAYOUT);
    // my range of positions in reverse sequence order, and my block inside it
    const int range = (B + parts - 1) / parts;
    const int p_begin = min(part * range, B), p_end = min(p_begin + range, B);
    const int per = (p_end - p_begin + kBuildThreads - 1) / kBuildThreads;
    const int r_begin = min(p_begin + tid * per, p_end), r_end = min(r_begin + per, p_end);
    int lo, len, mine = 0, ahead = 0;
    for (int r = tid; r < p_begin; r += kBuildThreads) ahead += chunks_of(resp_off, B - 1 - r, n_resp, lo, len, nullptr);
    for (int r = r_begin; r < r_end; ++r) mine += chunks_of(resp_off, B - 1 - r, n_resp, lo, len, status);
    int inc = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int y = __shfl_up(inc, off);
        if (lane >= off) inc += y;
        ahead += __shfl_xor(ahead, off);
    }
    if (lane == kWave - 1) s_wave[0][wave] = inc;
    if (lane == 0) s_wave[1][wave] = ahead;
    __syncthreads();
    int before = inc - mine, total = 0;
    for (int w = 0; w < kBuildThreads / kWave; ++w) {
        before += (w < wave ? s_wave[0][w] : 0) + s_wave[1][w];
        total += s_wave[0][w] + s_wave[1][w];
    }
    int next = before;                                          // processing index of my next sequence's last chunk
    for (int r = r_begin; r < r_end; ++r) {
        const int i = B - 1 - r;
        const int cnt = chunks_of(resp_off, i, n_resp, lo, len, nullptr);
        for (int c = cnt - 1; c >= 0; --c) {
            Chunk d;
            d.start = lo + c * kChunkTokens;
            d.pos_len = (c << 11) | (min(kChunkTokens, len - c * kChunkTokens) - 1);
            d.seg = i;
            d.after = cnt - 1 - c;
            const int w = next + (cnt - 1 - c);
            if (w < cap) chunks[w] = d;                         // overlapping sequences cannot overflow the list
        }
        next += cnt;
    }
    if (part == parts - 1 && tid == 0) {                        // the last range ends where the list ends
        if (total > cap) set_status(status, TPPO_STATUS_BAD_LAYOUT);
        n_chunks[0] = min(total, cap);
    }
}

}  // namespace tppo
