// tppo_egae: Extended GAE (Eq. (egae), Sec. 3.1) and returns R_t (Sec. 2.4) as
// one segmented reverse scan over the response-packed token array.
//
// Both recurrences are affine in the value carried in from the right, with a
// CONSTANT multiplier:
//   A_t = delta_t + (gamma*lambda) A_{t+1},   R_t = r_t + gamma R_{t+1},
// and restart at the last token of every sequence (where the bootstrap value of
// Sec. 3.1 enters delta).  So a run of n tokens acts on what is carried in as
// x -> m^n x + b, and only the b's have to be scanned.
//
// Work unit: one wavefront per tile of <= 1024 tokens of one sequence (plan.h),
// one tile per workgroup, no barriers.
//   * Loads and stores keep consecutive lanes on consecutive 16 bytes (the only
//     shape that streams at full rate), non-temporal, since every byte is
//     touched once.  A lane therefore owns, in each of 4 "slots", 4 consecutive
//     tokens; slot j is tokens 256 j .. 256 j + 255 of the tile.
//   * Lanes hold the 16-byte groups of a slot in REVERSE order (lane 0 the
//     highest addresses), so the right-to-left recurrence is a left-to-right
//     prefix scan over lanes, which the data-parallel primitives do without the
//     LDS crossbar: row_shr 1, 2, 4, 8, then row_bcast 15 and 31, each step one
//     fused multiply-add with the matching power of m^4.
//   * The four slots are chained by three scalar steps; the tile publishes
//     "value at my first token with nothing carried in" ({tag, float} words,
//     hi + lo of an fp64); a tile whose sequence continues to the right sums the
//     words of the (up to 64) following tiles with weights m^(1024 j), one per
//     lane.  Those words depend on no other tile, so there is no chain of waits.
//     Only a sequence of more than 65 tiles chains: there the 64th tile to the
//     right supplies its value with everything beyond included, which it
//     publishes once its own look-back is done.  The tiles waited for stand
//     earlier in the plan's list, which is sorted so that they started long
//     before (plan.h); they belong to lower workgroup ids in any case, so they
//     run or have run, and the wait is bounded besides.
//   * Second pass: replay each lane's 4-token runs from the value carried into
//     them, store A and R.
// HBM traffic is the algorithmic 16 B/token plus 16 B per tile of metadata.
//
// Arithmetic: inputs and outputs are fp32; TD residuals, partial sums and
// multipliers are fp64 (full rate on this chip).  With gamma*lambda close to 1 a
// sequence sums up to hundreds of thousands of residuals whose individual fp32
// rounding errors would add up (random walk) beyond 1e-5.
#include <math.h>
#include <stdlib.h>

#include <atomic>

#include "plan.h"

namespace tppo {

constexpr int kSpinLimit = 1 << 20;
#ifndef TPPO_EGAE_MIN_WAVES
#define TPPO_EGAE_MIN_WAVES 4
#endif
constexpr int kEgaeMinWaves = TPPO_EGAE_MIN_WAVES;   // wavefronts per SIMD the register allocation aims at
constexpr int kSlots = kTileTokens / 256;      // 16-byte groups per lane and array
static_assert(kSlots == 4, "a tile is four slots of 64 lanes x 4 tokens");

// wave-uniform powers of one recurrence's multiplier m, computed on the host
struct ScanConsts {
    double m;          // per token
    double q[6];       // (m^4)^(2^i): a step of 1, 2, 4, 8, 16, 32 lanes
    double q64;        // m^256: one slot
    double qtile;      // m^1024: one tile
};

static ScanConsts make_consts(double m) {
    ScanConsts s;
    s.m = m;
    for (int i = 0; i < 6; ++i) s.q[i] = pow(m, (double)(4 << i));
    s.q64 = pow(m, 256.0);
    s.qtile = pow(m, (double)kTileTokens);
    return s;
}

// data-parallel primitive move: lane i receives x of the lane the control word names; lanes without a
// source (start of a row, a row that row_mask leaves out) receive 0
template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_move(double x) {
    if constexpr (kRowMask == 0xF) {
        // every row is written: a lane without a source reads 0 by itself (bound_ctrl), and the destination
        // needs no initial value -- one instruction per half instead of two
        const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), kCtrl, 0xF, 0xF, true);
        const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), kCtrl, 0xF, 0xF, true);
        return __hiloint2double(hi, lo);
    } else {
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), kCtrl, kRowMask, 0xF, false);
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), kCtrl, kRowMask, 0xF, false);
        return __hiloint2double(hi, lo);
    }
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kWaveShr1 = 0x138, kRowBcast15 = 0x142, kRowBcast31 = 0x143;

__device__ __forceinline__ float wave_shr1(float x) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), kWaveShr1, 0xF, 0xF, true));
}

__device__ __forceinline__ double read_lane63(double x) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), 63),
                            __builtin_amdgcn_readlane(__double2loint(x), 63));
}

// per-lane powers of q = m^4: p = q^lane, w15 = q^(lane % 16 + 1), w31 = q^(lane % 32 + 1)
struct LaneWeights { double p, w15, w31; };

__device__ __forceinline__ LaneWeights lane_weights(const ScanConsts& s, int lane) {
    LaneWeights w = {1.0, 1.0, 1.0};
    if (s.m == 1.0) return w;                                    // wave-uniform
    double a = 1.0;                                              // q^(lane % 16)
#pragma unroll
    for (int i = 0; i < 4; ++i) a = ((lane >> i) & 1) ? a * s.q[i] : a;
    const double b = (lane & 16) ? a * s.q[4] : a;               // q^(lane % 32)
    w.w15 = a * s.q[0];
    w.w31 = b * s.q[0];
    w.p = (lane & 32) ? b * s.q[5] : b;
    return w;
}

// inclusive scan over the lanes of x_l = b_l + q x_{l-1}
__device__ __forceinline__ double lane_scan(double b, const ScanConsts& s, const LaneWeights& w) {
    b = fma(s.q[0], dpp_move<kRowShr1, 0xF>(b), b);
    b = fma(s.q[1], dpp_move<kRowShr2, 0xF>(b), b);
    b = fma(s.q[2], dpp_move<kRowShr4, 0xF>(b), b);
    b = fma(s.q[3], dpp_move<kRowShr8, 0xF>(b), b);
    b = fma(w.w15, dpp_move<kRowBcast15, 0xA>(b), b);            // lane 15 / 47 into rows 1 / 3
    b = fma(w.w31, dpp_move<kRowBcast31, 0xC>(b), b);            // lane 31 into rows 2 and 3
    return b;
}

// x^n for a non-negative integer n (0^0 = 1)
__device__ __forceinline__ double powi(double x, int n) {
    double r = 1.0;
    while (n > 0) {
        if (n & 1) r *= x;
        x *= x;
        n >>= 1;
    }
    return r;
}

// Four tagged words as loaded: the two doubles they carry; true when all four belong to this call.
__device__ __forceinline__ bool unpack_words(const unsigned long long (&w)[4], uint32_t tag, double& a, double& r) {
    a = (double)__uint_as_float((unsigned)w[0]) + (double)__uint_as_float((unsigned)w[1]);
    r = (double)__uint_as_float((unsigned)w[2]) + (double)__uint_as_float((unsigned)w[3]);
    return (uint32_t)(w[0] >> 32) == tag && (uint32_t)(w[1] >> 32) == tag && (uint32_t)(w[2] >> 32) == tag &&
           (uint32_t)(w[3] >> 32) == tag;
}

// Bounded wait for what a tile published (A hi, A lo, R hi, R lo).
__device__ __forceinline__ void wait_words(const unsigned long long* p, uint32_t tag, double& a, double& r,
                                           int32_t* status) {
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        // The word written last first: ONE load per round while the tile is not there yet.  (With all four
        // words polled every round, a list order in which most tiles wait took 154 us instead of 140: the
        // polls themselves were in the way.)
        const unsigned long long last = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(last >> 32) == tag) {
            const bool ok_a = poll(p, tag, a), ok_r = poll(p + 2, tag, r);
            if (ok_a && ok_r) return;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    set_status(status, TPPO_STATUS_TIMEOUT);
    a = 0.0;
    r = 0.0;
}

typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte access, 4-byte aligned

struct EgaeParams {
    const float* rewards;          // [n_resp], or with kTerminal the per-sequence terminal[B]
    const float* values;
    const int32_t* done;
    const float* bootstrap;
    float* adv;
    float* ret;
    void* plan;
    int32_t* status;
    int n_resp, B;
    uint32_t tag;
    double gamma;
    ScanConsts sa, sr;             // multipliers gamma*lambda (advantages) and gamma (returns)
};

// bits of x where keep, else zero: a select the compiler cannot turn into a branch, and one that never lets a
// NaN of a neighbouring sequence through (no multiplication by a mask)
__device__ __forceinline__ float keep_if(float x, bool keep) {
    return __int_as_float(__float_as_int(x) & (keep ? -1 : 0));
}

// A tile's inputs as loaded, with what the scalar side loads gave.
struct TileIn {
    float r[kSlots][4], v[kSlots][4];
    float side_next, side_last, side_boot, side_term;   // see issue_tile
    int side_done;
    unsigned long long early[4];   // the words of the tile this lane looks back at, as they stood when the tile began
    double look_a, look_r;         // what they carry
    bool look_ok;                  // ... if they were this call's
    Tile t;
    int pos;
};

// where lane `lane` of a tile looks: lane l at the tile l + 1 places to the right (l full tiles lie in between);
// if the sequence goes on beyond the 64th, that one's words with everything to its right included stand for
// the rest.  Lanes with nobody to look at are pointed at the last tile there is (own tile if none): a valid
// address whose contents they ignore.
__device__ __forceinline__ const unsigned long long* look_at(const Plan& pl, const Tile& t, int lane) {
    const bool rest = lane == kWave - 1 && t.after > kWave;
    return pl.scan_words + (int64_t)kScanWords * (t.slot() + min(lane + 1, t.after)) + (rest ? 4 : 0);
}

// What pass 1 leaves for pass 2 in registers.  The tokens' own values with nothing carried into their run of 4
// (32 floats per lane) wait in LDS meanwhile: the wavefront's private 8 KB, 16 bytes per lane and access,
// consecutive lanes on consecutive 16 bytes, no barrier (one wavefront per workgroup).  That keeps the kernel
// register count where 3 to 4 wavefronts fit a SIMD.
struct TileMid {
    double inc_a[kSlots], inc_r[kSlots];           // a run's value at its first token with nothing carried into the slot
    double tot_a[kSlots], tot_r[kSlots];           // a slot's value at its first token (wave-uniform)
};
typedef float lds_float4 __attribute__((ext_vector_type(4)));

// Issue the loads of tile `t` (list position `pos`).  The tile is tokens begin .. end - 1 of an aligned block of
// 1024 tokens of the arrays (plan.h); slot j, lane l holds the block's tokens k0 .. k0 + 3, k0 = 4 (64 j + 63 - l).
// Every lane with a token issues ONE 16-byte load per array: a group that straddles an end of the tile reads
// on into the neighbouring sequence (the surplus is zeroed later), and the one group that would read past the
// END OF THE ARRAY reads the array's last 16 bytes instead (moved into place later).  No branch
// and no wait separates the loads, so all of them are in flight together.  kTerminal: there is no reward array;
// the only reward is terminal[seq] on the last token of a finished sequence (Sec. 2.1: the rule-based reward
// arrives with the end of the response).
template <bool kTerminal>
__device__ __forceinline__ void issue_tile(TileIn& x, const Tile& t, const EgaeParams& p, const Plan& pl, int pos,
                                           int lane, int zero) {
    const float* __restrict__ rewards = p.rewards;
    const float* __restrict__ values = p.values;
    x.pos = pos;
    x.t = t;
    const int start = x.t.start, len = x.t.len(), seg = x.t.seg;
    const int base = x.t.base(), begin = x.t.begin(), end = begin + len;
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
        const int k0 = 4 * (64 * j + 63 - lane);
        float4u vv = {0.f, 0.f, 0.f, 0.f}, rr = {0.f, 0.f, 0.f, 0.f};
        if (k0 + 4 > begin && k0 < end) {
            const int at = min(base + k0, p.n_resp - 4);
            vv = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(values + at));
            if (!kTerminal) rr = __builtin_nontemporal_load(reinterpret_cast<const float4u*>(rewards + at));
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x.v[j][e] = vv[e];
            x.r[j][e] = rr[e];
        }
    }
    // What Eq. (TD) needs for the tile's last token, fetched unconditionally, every lane the same address, as
    // VECTOR loads that travel with the data (a scalar load that misses its cache was measured at three times
    // their latency, and pass 1 cannot start without these): V of the token after the tile, V(s_{l-1}), the
    // sequence's done flag, its bootstrap value, its terminal reward.  tile_front picks.  (`zero` is
    // opaque_zero(): without it the compiler turns loads from a uniform address into scalar ones.)
    const int seg_end = start + len;
    x.side_next = values[min(seg_end, p.n_resp - 1) + zero];
    x.side_last = values[seg_end - 1 + zero];
    x.side_done = p.done[seg + zero];
    x.side_boot = (p.bootstrap ? p.bootstrap + seg : values + start)[zero];
    x.side_term = kTerminal ? rewards[seg + zero] : 0.f;
    // The look-back's loads go out with the data's too, as ORDINARY cached loads.  The plan's list is sorted so
    // that the tiles looked at published long ago; their words then come from memory like any other data.  (A
    // load that must see other chiplets' latest stores -- device scope -- was measured at several times the
    // latency of a plain one.)  Should a lane get here before its tile published, the line it fetched may stay
    // in this chiplet's cache with the old contents; the tags say so, and tile_back then polls at device scope.
    // A tag is never reused, so stale words are never mistaken for this call's.
    const unsigned long long* look = look_at(pl, x.t, lane);
#pragma unroll
    for (int q = 0; q < 4; ++q) x.early[q] = __hip_atomic_load(look + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// Everything issue_tile asked for has arrived and is in its final form: the look-back's words are unpacked and
// every loaded register is pinned here, BEFORE any tile of the wavefront stores anything.  The memory counter
// of a wavefront retires in order, stores included: a wait for a load placed after a store -- the publication
// below, a tile's results -- also waits for that store, a full trip to memory.
__device__ __forceinline__ void settle_tile(TileIn& x, const EgaeParams& p) {
    x.look_ok = unpack_words(x.early, p.tag, x.look_a, x.look_r);
    asm volatile("" : "+v"(x.look_a), "+v"(x.look_r) : : "memory");
#pragma unroll
    for (int j = 0; j < kSlots; ++j)
        asm volatile("" : "+v"(x.v[j][0]), "+v"(x.v[j][1]), "+v"(x.v[j][2]), "+v"(x.v[j][3]), "+v"(x.r[j][0]),
                          "+v"(x.r[j][1]), "+v"(x.r[j][2]), "+v"(x.r[j][3]));
    asm volatile("" : "+v"(x.side_next), "+v"(x.side_last), "+v"(x.side_boot), "+v"(x.side_term), "+v"(x.side_done));
}

// Pass 1 of a tile, and the publication of its aggregate.  kFull: all 1024 tokens exist (every tile but a
// sequence's last): no masks -- straight-line code.
template <bool kTerminal, bool kFull>
__device__ __forceinline__ void tile_front(TileIn& x, TileMid& m, lds_float4* s_loc, const EgaeParams& p,
                                           const Plan& pl, int lane, const LaneWeights& wa,
                                           const LaneWeights& wr) {
    const double gamma = p.gamma, c = p.sa.m;
    const int n_resp = p.n_resp;
    const int base = x.t.base(), begin = kFull ? 0 : x.t.begin(), end = kFull ? kTileTokens : begin + x.t.len();
    // V(s_{t+1}) of the tile's last token: the next tile's first value, or the value of the state after the
    // sequence -- 0 for a finished one, else the bootstrap value, by default V(s_{l-1}) (Sec. 3.1)
    const bool fin = x.side_done != 0;
    const float v_end = x.t.after != 0 ? x.side_next : fin ? 0.f : p.bootstrap ? x.side_boot : x.side_last;
    const float terminal = (kTerminal && x.t.after == 0 && fin) ? x.side_term : 0.f;
    if (!kFull) {
        if (__builtin_expect(base + end > n_resp - 4, 0)) {         // wave-uniform: the array's last tile
#pragma unroll
            for (int j = 0; j < kSlots; ++j) {
                const int k0 = 4 * (64 * j + 63 - lane);
                const int sh = (k0 + 4 > begin && k0 < end) ? base + k0 - min(base + k0, n_resp - 4) : 0;
                float tv[4], tr[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    tv[e] = x.v[j][e];
                    tr[e] = x.r[j][e];
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x.v[j][e] = sh == 0 ? tv[e] : sh == 1 ? tv[(e + 1) & 3] : sh == 2 ? tv[(e + 2) & 3] : tv[(e + 3) & 3];
                    x.r[j][e] = sh == 0 ? tr[e] : sh == 1 ? tr[(e + 1) & 3] : sh == 2 ? tr[(e + 2) & 3] : tr[(e + 3) & 3];
                }
            }
        }
        // The block's tokens outside the tile become r = 0, V = 0, except that the place after the last token
        // takes the value that follows the tile: then Eq. (TD) needs no special case for the last token, and the
        // residuals of the padding are zeroed where they are computed.  (Padding to the RIGHT of the tile, only
        // in a sequence's last tile, sees no carry; padding to the left, only in a sequence's first tile, comes
        // after the tile in scan order and feeds nothing: the recurrences pass through the padding unharmed.)
#pragma unroll
        for (int j = 0; j < kSlots; ++j) {
            const int k0 = 4 * (64 * j + 63 - lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool in = k0 + e >= begin && k0 + e < end;
                x.r[j][e] = keep_if(x.r[j][e], in);
                x.v[j][e] = k0 + e == end ? v_end : keep_if(x.v[j][e], in);
            }
        }
    }
    if (kTerminal) {
#pragma unroll
        for (int j = 0; j < kSlots; ++j) {
            const int k0 = 4 * (64 * j + 63 - lane);
#pragma unroll
            for (int e = 0; e < 4; ++e) x.r[j][e] = keep_if(terminal, k0 + e == end - 1);
        }
    }
    // V of the token after each of my runs: my left neighbour's first value; for lane 0 the next slot's first
    // value (held by lane 63) or, after the last slot, the value after the tile
    float v_next_run[kSlots];
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
        const float from_lane = wave_shr1(x.v[j][0]);
        const float from_slot = j + 1 < kSlots
            ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x.v[j + 1][0]), 63)) : v_end;
        v_next_run[j] = lane == 0 ? from_slot : from_lane;
    }
    // Every run of 4 tokens as "values at its tokens with nothing carried in".  The chain is fp64; what a token
    // keeps for pass 2 is rounded to fp32 (a sum over <= 4 tokens, used once), what is carried on (the run's
    // value at its first token) stays fp64.  Then the runs are scanned over the lanes.
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
        double ba = 0.0, br = 0.0;
        if (kFull || (256 * j < end && 256 * (j + 1) > begin)) {    // wave-uniform: an empty slot stays zero
            const int k0 = 4 * (64 * j + 63 - lane);
            double vn = (double)v_next_run[j];
            lds_float4 la, lr;
#pragma unroll
            for (int e = 3; e >= 0; --e) {
                const double vk = (double)x.v[j][e], rk = (double)x.r[j][e];
                double delta = fma(gamma, vn, rk) - vk;             // Eq. (TD)
                if (!kFull) delta = (k0 + e >= begin && k0 + e < end) ? delta : 0.0;
                ba = fma(c, ba, delta);
                br = fma(gamma, br, rk);
                la[e] = (float)ba;
                lr[e] = (float)br;
                vn = vk;
            }
            s_loc[(2 * j) * kWave + lane] = la;
            s_loc[(2 * j + 1) * kWave + lane] = lr;
            ba = lane_scan(ba, p.sa, wa);
            br = lane_scan(br, p.sr, wr);
        }
        m.inc_a[j] = ba;
        m.inc_r[j] = br;
        m.tot_a[j] = read_lane63(ba);
        m.tot_r[j] = read_lane63(br);
    }
    // Take the look-back's words out of flight BEFORE anything is stored: the memory counter of a wavefront
    // retires in order, so a wait for these loads placed after the publication below would also wait for its
    // write-through stores, a full trip to memory.
    if (x.t.number() > 0) {                                         // somebody to my left will ask for the tile's value
        double ta = 0.0, tr = 0.0;
#pragma unroll
        for (int j = kSlots - 1; j >= 0; --j) {
            ta = fma(p.sa.q64, ta, m.tot_a[j]);
            tr = fma(p.sr.q64, tr, m.tot_r[j]);
        }
        if (lane == 0) {
            unsigned long long* words = &pl.scan_words[(int64_t)kScanWords * x.t.slot()];
            publish(words, p.tag, ta);
            publish(words + 2, p.tag, tr);
        }
    }
}

// The carry into a tile from the tiles to its right, pass 2, the stores.
template <bool kFull>
__device__ __forceinline__ void tile_back(const TileIn& x, const TileMid& m, const lds_float4* s_loc,
                                          const EgaeParams& p, const Plan& pl, int lane, const LaneWeights& wa,
                                          const LaneWeights& wr) {
    const Tile& t = x.t;
    const double gamma = p.gamma, c = p.sa.m;
    const int base = t.base(), begin = kFull ? 0 : t.begin(), end = kFull ? kTileTokens : begin + t.len(), after = t.after;
    double carry_a = 0.0, carry_r = 0.0;
    unsigned long long* words = &pl.scan_words[(int64_t)kScanWords * t.slot()];
    if (after != 0) {                                               // wave-uniform
        if (lane < after) {
            double ba = x.look_a, br = x.look_r;
            if (!x.look_ok)                                         // not there yet when the tile began: wait for it
                wait_words(look_at(pl, t, lane), p.tag, ba, br, p.status);
            carry_a = powi(p.sa.qtile, lane) * ba;
            carry_r = powi(p.sr.qtile, lane) * br;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            carry_a += __shfl_xor(carry_a, off);
            carry_r += __shfl_xor(carry_r, off);
        }
        if (t.number() >= kWave) {                                  // I am some tile's 64th: a full tile, since after != 0
            double ta = 0.0, tr = 0.0;
#pragma unroll
            for (int j = kSlots - 1; j >= 0; --j) {
                ta = fma(p.sa.q64, ta, m.tot_a[j]);
                tr = fma(p.sr.q64, tr, m.tot_r[j]);
            }
            if (lane == 0) {
                publish(words + 4, p.tag, fma(p.sa.qtile, carry_a, ta));
                publish(words + 6, p.tag, fma(p.sr.qtile, carry_r, tr));
            }
        }
    }
    // a token's value is what pass 1 kept for it plus m^(tokens to the run's end) times the value carried into
    // the run
    // (in fp32: what pass 1 kept is fp32 already and the result is rounded to fp32; the carry, an fp64 sum over
    // the whole rest of the sequence, is rounded once per run)
    const float pw_a[4] = {(float)p.sa.q[0], (float)(c * c * c), (float)(c * c), (float)c};
    const float pw_r[4] = {(float)p.sr.q[0], (float)(gamma * gamma * gamma), (float)(gamma * gamma), (float)gamma};
    float* __restrict__ adv = p.adv;
    float* __restrict__ ret = p.ret;
#pragma unroll
    for (int j = kSlots - 1; j >= 0; --j) {
        const int k0 = 4 * (64 * j + 63 - lane);
        if (kFull || (256 * j < end && 256 * (j + 1) > begin)) {
            const float xa = (float)fma(wa.p, carry_a, dpp_move<kWaveShr1, 0xF>(m.inc_a[j]));
            const float xr = (float)fma(wr.p, carry_r, dpp_move<kWaveShr1, 0xF>(m.inc_r[j]));
            const lds_float4 la = s_loc[(2 * j) * kWave + lane], lr = s_loc[(2 * j + 1) * kWave + lane];
            float4u oa, orr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                oa[e] = fmaf(pw_a[e], xa, la[e]);
                orr[e] = fmaf(pw_r[e], xr, lr[e]);
            }
            if (kFull || (k0 >= begin && k0 + 4 <= end)) {
                __builtin_nontemporal_store(oa, reinterpret_cast<float4u*>(adv + base + k0));
                __builtin_nontemporal_store(orr, reinterpret_cast<float4u*>(ret + base + k0));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (k0 + e >= begin && k0 + e < end) {
                        adv[base + k0 + e] = oa[e];
                        ret[base + k0 + e] = orr[e];
                    }
                }
            }
        }
        carry_a = fma(p.sa.q64, carry_a, m.tot_a[j]);
        carry_r = fma(p.sr.q64, carry_r, m.tot_r[j]);
    }
}

// Schedule: one wavefront per workgroup, kTilesPerWave consecutive list positions per wavefront; the hardware's
// dispatcher is the load balancer, and it starts workgroups in index order: the tiles a tile may have to wait
// for stand earlier in the list, so they run or have run (or are this wavefront's own earlier tile), and they
// never wait before they publish.  All loads of all the wavefront's tiles go out first, then the tiles are
// worked through one after the other: the start of a wavefront, the trip to memory and the drain of the
// stores are paid once per kTilesPerWave tiles, and no load ever waits behind a store.
// Measured on the 40 M-token long-CoT batch: 1 tile per wavefront 135 us (4 wavefronts per SIMD), 2 tiles 149 us
// (3 per SIMD), 3 tiles 173 us (2 per SIMD) -- what a second tile saves in start-up and drain it loses in
// wavefronts per SIMD, and a tile that is worked on later publishes later.  Wavefronts that stay and walk the
// list in a loop: every tile then waits for the stores of the one before it; 150 us.
#ifndef TPPO_EGAE_TILES
#define TPPO_EGAE_TILES 1
#endif
constexpr int kTilesPerWave = TPPO_EGAE_TILES;

template <bool kTerminal>
__device__ __forceinline__ void run_tile(TileIn& x, lds_float4* s_loc, const EgaeParams& p, const Plan& pl, int lane,
                                         const LaneWeights& wa, const LaneWeights& wr) {
    TileMid mid;
    if (x.t.len() == kTileTokens) {
        tile_front<kTerminal, true>(x, mid, s_loc, p, pl, lane, wa, wr);
        tile_back<true>(x, mid, s_loc, p, pl, lane, wa, wr);
    } else {
        tile_front<kTerminal, false>(x, mid, s_loc, p, pl, lane, wa, wr);
        tile_back<false>(x, mid, s_loc, p, pl, lane, wa, wr);
    }
}

template <bool kTerminal>
__global__ __launch_bounds__(kWave, kEgaeMinWaves) void egae_scan_kernel(EgaeParams p) {
    __shared__ lds_float4 s_loc[2 * kSlots * kWave];
    const int lane = threadIdx.x;
    const int pos0 = blockIdx.x * kTilesPerWave;
    // The descriptors are asked for before anything is known about the plan -- their place depends on the
    // plan's address alone, and the caller guarantees a buffer that holds them -- so that they travel together
    // with the header instead of after it.  As vector loads: the wavefront waits for them, and a scalar load
    // that misses is several times slower.
    const int zero = opaque_zero();
    const Tile* list = reinterpret_cast<const Tile*>(static_cast<const char*>(p.plan) + 256);
    tile_bits raw[kTilesPerWave];
#pragma unroll
    for (int h = 0; h < kTilesPerWave; ++h) raw[h] = fetch_tile(list + pos0 + h, zero);
    const Plan pl = plan_open(p.plan);
    const int n_tiles = load_uniform(&pl.hdr->n_tiles);
    if (load_uniform(&pl.hdr->B) != p.B || load_uniform(&pl.hdr->n_resp) != p.n_resp || n_tiles > pl.cap ||
        pl.cap < p.n_resp / kTileTokens + p.B + 1) {                // a plan built for another batch
        if (pos0 == 0 && lane == 0) set_status(p.status, TPPO_STATUS_BAD_LAYOUT);
        return;
    }
    if (pos0 >= n_tiles) return;                                    // the list is shorter than its capacity
    TileIn x[kTilesPerWave];
    bool live[kTilesPerWave];
#pragma unroll
    for (int h = 0; h < kTilesPerWave; ++h) {
        const Tile t = uniform_tile(raw[h]);
        live[h] = pos0 + h < n_tiles;
        if (live[h] && !tile_valid(t, p.n_resp, p.B, pl.cap)) {
            if (lane == 0) set_status(p.status, TPPO_STATUS_BAD_LAYOUT);
            live[h] = false;
        }
        if (live[h]) issue_tile<kTerminal>(x[h], t, p, pl, pos0 + h, lane, zero);
    }
    const LaneWeights wa = lane_weights(p.sa, lane), wr = lane_weights(p.sr, lane);    // while the loads fly
#pragma unroll
    for (int h = 0; h < kTilesPerWave; ++h)
        if (live[h]) settle_tile(x[h], p);
#pragma unroll
    for (int h = 0; h < kTilesPerWave; ++h)
        if (live[h]) run_tile<kTerminal>(x[h], s_loc, p, pl, lane, wa, wr);
}

// Batches of fewer than four tokens (the streaming kernel's 16-byte accesses need four): one thread per
// sequence walks it token by token, straight from Eq. (TD) and the two recurrences.
template <bool kTerminal>
__global__ __launch_bounds__(256) void egae_tiny_kernel(const float* __restrict__ rewards, const float* __restrict__ values,
                                                        const int32_t* __restrict__ resp_off, const int32_t* __restrict__ done,
                                                        const float* __restrict__ bootstrap, int B, int n_resp, double gamma,
                                                        double c, float* __restrict__ adv, float* __restrict__ ret,
                                                        int32_t* status) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < B; i += gridDim.x * blockDim.x) {
        const int lo = resp_off[i], hi = resp_off[i + 1];
        if (lo < 0 || hi < lo || hi > n_resp) {
            set_status(status, TPPO_STATUS_BAD_LAYOUT);
            continue;
        }
        if (hi == lo) continue;
        const bool fin = done[i] != 0;
        double v_next = fin ? 0.0 : (double)(bootstrap ? bootstrap[i] : values[hi - 1]);
        double a = 0.0, r = 0.0;
        for (int t = hi - 1; t >= lo; --t) {
            const double rk = kTerminal ? ((t == hi - 1 && fin) ? (double)rewards[i] : 0.0) : (double)rewards[t];
            const double vk = (double)values[t];
            a = fma(c, a, fma(gamma, v_next, rk) - vk);
            r = fma(gamma, r, rk);
            adv[t] = (float)a;
            ret[t] = (float)r;
            v_next = vk;
        }
    }
}

}  // namespace tppo

extern "C" size_t tppo_egae_workspace_bytes(int64_t n_resp, int64_t B) {
    if (n_resp <= 0 || B <= 0) return 256;
    return tppo::plan_bytes_for(tppo::plan_max_tiles(n_resp, B));
}

namespace tppo {
// `rewards` is the dense [n_resp] array, or with terminal_mode the per-sequence terminal[B] array.
// plan != NULL: a plan of this layout, built earlier on the same stream; else one is built in `workspace`.
static int egae_launch(const float* rewards, bool terminal_mode, const float* values, const int32_t* resp_off,
                       const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                       float gamma, float lambda, float* adv, float* ret, void* workspace,
                       size_t workspace_bytes, void* plan, int32_t* status, void* stream) {
    if (B < 0 || n_resp < 0 || n_resp > INT32_MAX - kTileTokens || B > INT32_MAX / 4) return TPPO_ERR_SIZE;
    if (!(gamma >= 0.f && gamma <= 1.f) || !(lambda >= 0.f && lambda <= 1.f)) return TPPO_ERR_PARAM;
    if (n_resp == 0) return TPPO_OK;
    if (B == 0) return TPPO_ERR_SIZE;
    if (!rewards || !values || !resp_off || !done || !adv || !ret) return TPPO_ERR_NULL;
    int64_t cap64 = plan_max_tiles(n_resp, B);
    if (cap64 > INT32_MAX / 8) return TPPO_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan) {
        if (!is_aligned(plan, 256)) return TPPO_ERR_WORKSPACE;
    } else if (!workspace || !is_aligned(workspace, 256) || workspace_bytes < tppo_egae_workspace_bytes(n_resp, B)) {
        return TPPO_ERR_WORKSPACE;
    }
    if (n_resp < 4) {
        const int groups = (int)((B + 255) / 256 < 1024 ? (B + 255) / 256 : 1024);
        const double g = (double)gamma, c = (double)gamma * (double)lambda;
        if (terminal_mode)
            hipLaunchKernelGGL(egae_tiny_kernel<true>, dim3(groups), dim3(256), 0, s, rewards, values, resp_off, done,
                               bootstrap, (int)B, (int)n_resp, g, c, adv, ret, status);
        else
            hipLaunchKernelGGL(egae_tiny_kernel<false>, dim3(groups), dim3(256), 0, s, rewards, values, resp_off, done,
                               bootstrap, (int)B, (int)n_resp, g, c, adv, ret, status);
        return launch_result();
    }
    if (!plan) {
        if (launch_plan_build(resp_off, nullptr, done, B, n_resp, cap64, workspace, status, s) != TPPO_OK) return TPPO_ERR_LAUNCH;
        plan = workspace;
    }
    EgaeParams p;
    p.rewards = rewards; p.values = values; p.done = done; p.bootstrap = bootstrap;
    p.adv = adv; p.ret = ret; p.plan = plan; p.status = status;
    p.n_resp = (int)n_resp; p.B = (int)B;
    p.tag = next_call_tag();
    p.gamma = (double)gamma;
    p.sa = make_consts((double)gamma * (double)lambda);
    p.sr = make_consts((double)gamma);
    // one wavefront per kTilesPerWave tiles; the list may be shorter than its capacity: the surplus exits at once
    const unsigned groups = (unsigned)((cap64 + kTilesPerWave - 1) / kTilesPerWave);
    if (terminal_mode) hipLaunchKernelGGL(egae_scan_kernel<true>, dim3(groups), dim3(kWave), 0, s, p);
    else hipLaunchKernelGGL(egae_scan_kernel<false>, dim3(groups), dim3(kWave), 0, s, p);
    return launch_result();
}
}  // namespace tppo

extern "C" int tppo_egae(const float* rewards, const float* values, const int32_t* resp_off,
                         const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                         float gamma, float lambda, float* adv, float* ret, void* workspace,
                         size_t workspace_bytes, void* plan, int32_t* status, void* stream) {
    return tppo::egae_launch(rewards, false, values, resp_off, done, bootstrap, B, n_resp, gamma, lambda, adv,
                             ret, workspace, workspace_bytes, plan, status, stream);
}

// ---------------------------------------------------------------------------------------------------------
// tppo_egae_static: tppo_egae for callers that may not allocate.  The plan is built in a fixed array that is
// part of the library's image on every GPU it runs on.
namespace tppo {
constexpr int64_t kStaticTiles = 47872;                            // plan capacity of the array, in tiles
constexpr size_t kStaticBytes = plan_bytes_for(kStaticTiles);      // 5.27 MiB
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// The array's address on the current device.  In host code `scratch` is only a handle: the address has to be
// asked for, once per device and with that device current (every GPU holds its own copy at its own address).
static void* static_plan_memory() {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> known[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* ptr = known[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return nullptr;
    }
    known[dev].store(ptr, std::memory_order_release);            // (two threads racing here store the same value)
    return ptr;
}
}  // namespace tppo

extern "C" int64_t tppo_egae_static_max_tiles(void) { return tppo::kStaticTiles; }

extern "C" int tppo_egae_static(const float* rewards, const float* values, const int32_t* resp_off,
                                const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                                float gamma, float lambda, float* adv, float* ret, int32_t* status, void* stream) {
    using namespace tppo;
    if (B < 0 || n_resp < 0) return TPPO_ERR_SIZE;
    if (n_resp / kTileTokens + B + 1 > kStaticTiles) return TPPO_ERR_SIZE;        // more tiles than the array holds
    void* mem = static_plan_memory();
    if (!mem) return TPPO_ERR_LAUNCH;
    return egae_launch(rewards, false, values, resp_off, done, bootstrap, B, n_resp, gamma, lambda, adv, ret, mem,
                       kStaticBytes, nullptr, status, stream);
}

extern "C" int tppo_egae_terminal(const float* terminal_reward, const float* values, const int32_t* resp_off,
                                  const int32_t* done, const float* bootstrap, int64_t B, int64_t n_resp,
                                  float gamma, float lambda, float* adv, float* ret, void* workspace,
                                  size_t workspace_bytes, void* plan, int32_t* status, void* stream) {
    return tppo::egae_launch(terminal_reward, true, values, resp_off, done, bootstrap, B, n_resp, gamma, lambda,
                             adv, ret, workspace, workspace_bytes, plan, status, stream);
}
