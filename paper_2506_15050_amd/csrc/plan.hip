// tppo_plan_build: the work plan of a batch layout (plan.h), built once and
// handed to tppo_egae*, tppo_ppo_losses and tppo_ppo_losses_backward so that
// none of them has to cut the batch into tiles again.  tppo_select builds the
// same plan as a by-product of the token filter (Sec. 3.2).
#include <atomic>

#include "plan.h"

namespace tppo {

uint32_t next_call_tag() {
    static std::atomic<uint32_t> counter{0};
    uint32_t t = counter.fetch_add(1, std::memory_order_relaxed) + 1;
    if (t == 0) t = counter.fetch_add(1, std::memory_order_relaxed) + 1;   // 0 means "never written"
    return t;
}

int device_compute_units() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> known[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return 0;
    if (dev < kMaxDevices) {
        const int v = known[dev].load(std::memory_order_relaxed);
        if (v > 0) return v;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (dev < kMaxDevices && cus > 0) known[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

__device__ __forceinline__ int window_of(const int32_t* __restrict__ resp_off, int i, int n_resp, int& lo,
                                         int32_t* status) {
    lo = resp_off[i];
    const int hi = resp_off[i + 1];
    if (lo < 0 || hi < lo || hi > n_resp) {
        if (status) set_status(status, TPPO_STATUS_BAD_LAYOUT);
        return 0;
    }
    return hi - lo;
}

// Tiles are cut at multiples of kTileTokens of the response-packed INDEX, not of the position inside the
// sequence: every tile but a sequence's first and last is then a 4 KiB-aligned block of each array (given
// aligned arrays), which is worth 10-15 % to a streaming kernel on this chip -- a wavefront's 1 KiB access
// that straddles 128-byte lines costs an extra line each time.  The price is up to one more (short) tile per
// sequence.
__device__ __forceinline__ int window_tiles(int lo, int len) {
    return len > 0 ? ((lo + len - 1) / kTileTokens) - (lo / kTileTokens) + 1 : 0;
}

__device__ __forceinline__ int wave_max(int x) {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) x = max(x, __shfl_xor(x, off));
    return __builtin_amdgcn_readfirstlane(x);
}

// The tile that begins a frame describes the frame.  If its sequence ends inside the frame, the builder also
// looks up the sequence that follows (skipping at most kSkipEmpty empty ones; beyond that the consumers look
// for themselves).
constexpr int kSkipEmpty = 64;
__device__ __forceinline__ void note_frame(const Plan& pl, const Tile& d, int lo, int len, const int32_t* resp_off,
                                           const int32_t* keep_len, const int32_t* done, int B, int n_resp, int keep,
                                           bool fin) {
    if ((d.start & (kTileTokens - 1)) != 0) return;
    const int f = d.start / kTileTokens;
    if (f >= pl.cap) return;
    const int end = lo + len;
    FrameDesc x = {d.seg, end, keep_len ? lo + min(max(keep, 0), len) : lo, fin ? 1 : 0, d.seg, end, end, 0};
    if (end < d.start + kTileTokens && end < n_resp) {
        int j = d.seg + 1;
        for (int step = 0; step < kSkipEmpty && j < B && resp_off[j + 1] <= end; ++step) ++j;
        if (j < B && resp_off[j] == end && resp_off[j + 1] > end && resp_off[j + 1] <= n_resp) {
            const int len2 = resp_off[j + 1] - end;
            x.seg2 = j;
            x.end2 = end + len2;
            x.pol_end2 = keep_len ? end + min(max(keep_len[j], 0), len2) : end;
            x.fin2 = (keep_len && done[j] != 0) ? 1 : 0;
        }
    }
    pl.frames[f] = x;
}

__device__ __forceinline__ Tile make_tile(int seg, int lo, int len, int tiles, int after) {
    const int c = tiles - 1 - after;
    const int block = lo / kTileTokens + c;                             // which aligned block of the arrays
    const int first = max(lo, block * kTileTokens), last = min(lo + len, (block + 1) * kTileTokens);
    Tile d;
    d.start = first;
    d.pos_len = (c << kTileShift) | (last - first - 1);
    d.seg = seg;
    d.after = after;
    return d;
}

// Workgroups 0 .. parts-1 build the list: workgroup `part` owns a contiguous range of the sequences and,
// inside it, thread t a contiguous block.  A tile of level l goes to
//   (tiles of lower levels, whole batch) + (level-l tiles of the sequences before the range)
//   + (level-l tiles of the range's wavefronts before mine) + (its rank inside the wavefront).
// Every builder counts the first two terms by itself, from offsets that sit in the cache -- cheaper than a
// second launch.  All counting is by ballot, level by level, in loops that run as deep as the longest
// sequence the wavefront is looking at: the code stays small (a kernel that runs once per batch pays for
// every instruction-cache line it touches; the fully unrolled form of this one took 20 us on 32 sequences)
// and short batches cost little.  Inside a level the order is whatever the ballots give; only the level order
// matters.  Workgroup `parts` counts the two token sets meanwhile; the remaining workgroups zero the tagged
// words.
__global__ __launch_bounds__(kBuildThreads) void plan_build_kernel(const int32_t* __restrict__ resp_off,
                                                                   const int32_t* __restrict__ keep_len,
                                                                   const int32_t* __restrict__ done, int B,
                                                                   int n_resp_arg, int cap, int parts, void* plan_raw,
                                                                   int32_t* status) {
    constexpr int kWaves = kBuildThreads / kWave;
    __shared__ long long s_cnt[2][kWaves];
    // per wavefront and level: tiles of the whole batch [0], of the sequences before my range [1], of my range [2]
    // ([.][.][kLevels]: tiles beyond the sorted levels)
    __shared__ int s_cnt3[3][kWaves][kLevels + 1];
    __shared__ int s_sum[2][kLevels + 1];
    __shared__ int s_first[kLevels + 1];                   // list position of the range's first tile of a level
    __shared__ int s_total;
    const Plan pl = plan_view(plan_raw, cap);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int block = blockIdx.x;
    if (block > parts) {                                   // zero the tagged words
        const int64_t words = plan_words(cap);
        for (int64_t i = (int64_t)(block - parts - 1) * kBuildThreads + tid; i < words;
             i += (int64_t)(gridDim.x - parts - 1) * kBuildThreads)
            pl.scan_words[i] = 0ull;
        return;
    }
    if (block == parts) {                                  // sizes of the two token sets, from the metadata alone
        long long np = 0, nv = 0;
        if (keep_len) {
            for (int i = tid; i < B; i += kBuildThreads) {
                const int win = max(resp_off[i + 1] - resp_off[i], 0);
                np += min(max(keep_len[i], 0), win);
                nv += done[i] != 0 ? win : 0;
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            np += __shfl_down(np, off);
            nv += __shfl_down(nv, off);
        }
        if (lane == 0) {
            s_cnt[0][wave] = np;
            s_cnt[1][wave] = nv;
        }
        __syncthreads();
        if (tid == 0) {
            np = nv = 0;
            for (int w = 0; w < kWaves; ++w) {
                np += s_cnt[0][w];
                nv += s_cnt[1][w];
            }
            pl.hdr->n_policy = np;
            pl.hdr->n_value = nv;
            pl.hdr->has_sets = keep_len ? 1 : 0;
        }
        return;
    }
    const int part = block;
    const int n_resp = n_resp_arg >= 0 ? n_resp_arg : resp_off[B];
    if (part == 0 && tid == 0 && (resp_off[0] != 0 || resp_off[B] != n_resp)) set_status(status, TPPO_STATUS_BAD_LAYOUT);
    const int range = (B + parts - 1) / parts;
    const int p_begin = min(part * range, B), p_end = min(p_begin + range, B);
    const int per = (p_end - p_begin + kBuildThreads - 1) / kBuildThreads;
    const int i_begin = min(p_begin + tid * per, p_end), i_end = min(i_begin + per, p_end);
    int lo;
    for (int k = tid; k < 3 * kWaves * (kLevels + 1); k += kBuildThreads) (&s_cnt3[0][0][0])[k] = 0;
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1;          // lanes before mine
    // wave-wide: add, per level, the lanes whose sequence has a tile there to row `row` of the counters
    auto count_levels = [&](int which, int tiles) {
        const int deepest = wave_max(tiles);
        for (int l = 0; l < min(deepest, kLevels); ++l) {
            const int c = __popcll(__ballot(tiles > l));
            if (lane == 0) s_cnt3[which][wave][l] += c;
        }
        if (deepest > kLevels) {                                    // tiles beyond the sorted levels
            int extra = max(tiles - kLevels, 0);
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) extra += __shfl_xor(extra, off);
            if (lane == 0) s_cnt3[which][wave][kLevels] += extra;
        }
    };
    // whole batch (0) and the sequences before my range (1): every wavefront its share, strided
    for (int i0 = wave * kWave; i0 < B; i0 += kBuildThreads) {
        const int i = i0 + lane;
        int tiles = 0;
        if (i < B) {
            const int len = window_of(resp_off, i, n_resp, lo, nullptr);
            tiles = window_tiles(lo, len);
        }
        count_levels(0, tiles);
        if (i0 < p_begin) count_levels(1, i < p_begin ? tiles : 0);
    }
    // my range (2): thread t owns sequences i_begin .. i_end - 1; the wavefront handles one of each at a time
    for (int k = 0; k < per; ++k) {
        const int i = i_begin + k;
        int tiles = 0;
        if (i < i_end) {
            const int len = window_of(resp_off, i, n_resp, lo, status);
            tiles = window_tiles(lo, len);
        }
        count_levels(2, tiles);
    }
    __syncthreads();
    if (tid < 2 * (kLevels + 1)) {                                  // totals over the wavefronts
        const int which = tid / (kLevels + 1), l = tid % (kLevels + 1);
        int sum = 0;
        for (int w = 0; w < kWaves; ++w) sum += s_cnt3[which][w][l];
        s_sum[which][l] = sum;
    } else if (tid >= 128 && tid <= 128 + kLevels) {                // another wavefront: my range's counts into offsets
        const int l = tid - 128;
        int run = 0;
        for (int w = 0; w < kWaves; ++w) {
            const int x = s_cnt3[2][w][l];
            s_cnt3[2][w][l] = run;
            run += x;
        }
    }
    __syncthreads();
    if (tid <= kLevels) {                                           // where each level starts for this range
        int base = 0;
        for (int l = 0; l < tid; ++l) base += s_sum[0][l];
        s_first[tid] = base + s_sum[1][tid];
        if (tid == kLevels) s_total = base + s_sum[0][kLevels];
    }
    __syncthreads();
    // Emission, in the same order as the count of my range.  s_cnt3[2][wave][l] is the wavefront's running
    // offset inside level l (wave-private from here on).
    for (int k = 0; k < per; ++k) {
        const int i = i_begin + k;
        int tiles = 0, len = 0, keep = 0;
        bool fin = false;
        if (i < i_end) {
            len = window_of(resp_off, i, n_resp, lo, nullptr);
            tiles = window_tiles(lo, len);
            if (keep_len && tiles > 0) {
                keep = keep_len[i];
                fin = done[i] != 0;
            }
        }
        const int deepest = wave_max(tiles);
        for (int l = 0; l < min(deepest, kLevels); ++l) {
            const unsigned long long has = __ballot(tiles > l);
            const int at = s_first[l] + s_cnt3[2][wave][l] + __popcll(has & below);
            if (tiles > l && at < cap) {                            // (invalid offsets cannot overflow the list)
                const Tile d = make_tile(i, lo, len, tiles, l);
                pl.tiles[at] = d;
                note_frame(pl, d, lo, len, resp_off, keep_len, done, B, n_resp, keep, fin);
            }
            if (lane == 0) s_cnt3[2][wave][l] += __popcll(has);
        }
        if (deepest > kLevels) {                                    // a sequence's deeper tiles stay together
            const int extra = max(tiles - kLevels, 0);
            int inc = extra;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const int y = __shfl_up(inc, off);
                if (lane >= off) inc += y;
            }
            int at = s_first[kLevels] + s_cnt3[2][wave][kLevels] + inc - extra;
            for (int l = kLevels; l < tiles; ++l, ++at) {
                if (at < cap) {
                    const Tile d = make_tile(i, lo, len, tiles, l);
                    pl.tiles[at] = d;
                    note_frame(pl, d, lo, len, resp_off, keep_len, done, B, n_resp, keep, fin);
                }
            }
            const int total = __shfl(inc, kWave - 1);
            if (lane == 0) s_cnt3[2][wave][kLevels] += total;
        }
    }
    if (part == parts - 1 && tid == 0) {
        const int total = s_total;
        if (total > cap) set_status(status, TPPO_STATUS_BAD_LAYOUT);
        pl.hdr->n_tiles = min(total, cap);
        pl.hdr->B = B;
        pl.hdr->n_resp = n_resp;
        pl.hdr->cap = cap;
    }
}

int launch_plan_build(const int32_t* resp_off, const int32_t* keep_len, const int32_t* done, int64_t B,
                      int64_t n_resp, int64_t cap, void* plan_raw, int32_t* status, hipStream_t s) {
    const int parts = build_parts(B);
    int64_t zero_groups = (plan_words(cap) + kBuildThreads * 8 - 1) / (kBuildThreads * 8);
    zero_groups = zero_groups < 1 ? 1 : zero_groups > 4096 ? 4096 : zero_groups;
    hipLaunchKernelGGL(plan_build_kernel, dim3(parts + 1 + (int)zero_groups), dim3(kBuildThreads), 0, s, resp_off,
                       keep_len, done, (int)B, (int)(n_resp < 0 ? -1 : n_resp), (int)cap, parts, plan_raw, status);
    return launch_result();
}

}  // namespace tppo

extern "C" size_t tppo_plan_bytes(int64_t n_resp, int64_t B) {
    if (n_resp < 0 || B < 0) return 256;
    return tppo::plan_bytes_for(tppo::plan_max_tiles(n_resp, B));
}

extern "C" int tppo_plan_build(const int32_t* resp_off, const int32_t* keep_len, const int32_t* done, int64_t B,
                               int64_t n_resp, void* plan, size_t plan_bytes, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kTileTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (n_resp > 0 && B == 0) return TPPO_ERR_SIZE;
    if (!resp_off || (B > 0 && !done)) return TPPO_ERR_NULL;
    if (plan_max_tiles(n_resp, B) > INT32_MAX / 8) return TPPO_ERR_SIZE;
    if (!plan || !is_aligned(plan, 256) || plan_bytes < tppo_plan_bytes(n_resp, B)) return TPPO_ERR_WORKSPACE;
    return launch_plan_build(resp_off, keep_len, done, B, n_resp, plan_max_tiles(n_resp, B), plan, status,
                             static_cast<hipStream_t>(stream));
}
