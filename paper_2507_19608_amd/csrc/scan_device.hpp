// Device code of the delta matrix construction (Sec. II-C Eq. 2-3; Sec. III-A strategy 3) and of the compaction of
// surviving entries per key column, shared by the stand-alone kernels and by the fused short-prompt prefill kernel.
#pragma once
#include "common.hpp"

namespace da {

// Eq. 2-3 over rows t0 .. t1 - 1 of one unit for the 64 channels c = 64 * channel_wave + lane, by one wave.
//   first   : the rows start a sequence or continue one: row t0 is then the basis row (kept whole), or, with `init`
//             given, the first row after the reference key init[c]
//   !first  : the scan starts from `start` (the held value before row t0)
// kFinal: mask words, reference keys (Hp) are written and surviving entries counted into *count; otherwise only the
// held value at the end is returned (a speculative pass).
template <typename T, bool kFinal>
__device__ __forceinline__ float scan_rows(const T *__restrict__ Kp, T *__restrict__ Hp, uint32_t *__restrict__ Mp,
                                           int d, int c, int lane, int t0, int t1, bool first, const T *init_row,
                                           float start, float theta, unsigned long long *count) {
    const bool active = c < d;
    const int wpr = d >> 5;
    const bool writer = active && ((lane & 31) == 0);
    const int word = c >> 5;
    const int cs = active ? c : 0;
    // The held value is always a verbatim copy of a key element (or of the incoming state): its stored form is
    // carried along beside the binary32 value the comparison uses, so that storing a reference key converts nothing.
    float held = start;
    T held_raw = from_f32<T>(start);
    unsigned long long cnt = 0;
    int t = t0;
    if (first && init_row) {   // the rows continue a sequence: its reference key is the incoming state
        held_raw = init_row[cs];
        held = to_f32(held_raw);
    } else if (first) {        // row t0 is the basis: kept whole
        held_raw = Kp[(size_t)t0 * d + cs];
        held = to_f32(held_raw);
        if (kFinal) {
            if (active) Hp[(size_t)t0 * d + c] = held_raw;
            if (writer) Mp[(size_t)t0 * wpr + word] = 0xffffffffu;
            cnt = __popcll(__ballot(active));
        }
        t = t0 + 1;
    }
    // Rows in batches of U; two register sets alternate, the next batch is requested before the current one is
    // worked on (loads past the end are clamped to the last row and never used), so that a batch's memory
    // latency is hidden behind the previous batch's arithmetic instead of being paid once per batch.  The mask
    // words of a batch are collected in registers (lane u of each half keeps the word of row u) and stored once.
    constexpr int U = 16;
    auto load_batch = [&](T (&k)[U], int tb) {
#pragma unroll
        for (int u = 0; u < U; ++u) k[u] = Kp[(size_t)min(tb + u, t1 - 1) * d + cs];
    };
    auto work_batch = [&](const T (&k)[U], int tb) {
        uint32_t my_word = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float kf = to_f32(k[u]);
            const float diff = kf - held;                    // Eq. 2 condition in binary32
            const bool fire = active && (fabsf(diff) > theta);
            held = fire ? kf : held;                          // Eq. 3
            held_raw = fire ? k[u] : held_raw;
            if (kFinal) {
                const uint64_t b = __ballot(fire);
                my_word = ((lane & 31) == u) ? (uint32_t)(b >> (lane & 32)) : my_word;
                if (active) Hp[(size_t)(tb + u) * d + c] = held_raw;
                cnt += __popcll(b);
            }
        }
        if (kFinal && active && (lane & 31) < U) Mp[(size_t)(tb + (lane & 31)) * wpr + word] = my_word;
    };
    if (t + U <= t1) {
        T ka[U], kb[U];
        load_batch(ka, t);
        while (t + U <= t1) {
            load_batch(kb, t + U);
            work_batch(ka, t);
            t += U;
            if (t + U > t1) break;
            load_batch(ka, t + U);
            work_batch(kb, t);
            t += U;
        }
    }
    for (; t < t1; ++t) {
        const T kr = Kp[(size_t)t * d + cs];
        const float k = to_f32(kr);
        const bool fire = active && (fabsf(k - held) > theta);
        held = fire ? k : held;
        held_raw = fire ? kr : held_raw;
        if (kFinal) {
            const uint64_t b = __ballot(fire);
            if (writer) Mp[(size_t)t * wpr + word] = (uint32_t)(b >> (lane & 32));
            if (active) Hp[(size_t)t * d + c] = held_raw;
            cnt += __popcll(b);
        }
    }
    if (kFinal) *count = cnt;
    return held;
}

// Compaction of one key column j of a unit by one wave: ballot + prefix count turn the mask row into a dense list of
// (channel, delta) pairs in EntryChunk form (see emit_entries_kernel); blk_cnt[slot_in_block] receives the chunk count.
// In two steps, so that a wave can have the next column's inputs in flight while it works on this one (a column is
// a short chain of dependent memory round trips; one column at a time is latency bound):
//   load_column    every input of the column: the lane's mask word, key and previous reference key of each 64-channel
//                  pass (all loads unconditional, indices clamped into the arrays)
//   finish_column  the compaction proper
// K0, H0, M0: row 0 of the unit's keys, reference keys and mask words (global memory or an LDS copy);
// ents0, counts0, nch0: the unit's first entry chunk, count and chunk-count slot (global).
constexpr int kMaxPass = 4;                                   // 64-channel passes of a column: head_dim <= 256
struct ColumnIn {
    float k[kMaxPass], held[kMaxPass];
    uint32_t word[kMaxPass];
};

template <typename T>
__device__ __forceinline__ void load_column(ColumnIn &in, const T *K0, const T *H0, const uint32_t *M0, int n, int d,
                                            int lane, int j) {
    const size_t row = (size_t)min(j, n - 1);                 // columns past the end are never finished
    const T *Kp = K0 + row * d;
    const T *Hprev = H0 + (row - (row > 0 ? 1 : 0)) * d;
    const uint32_t *Mp = M0 + row * (d >> 5);
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        const int c = min(p * kWave + lane, d - 1);
        in.word[p] = Mp[c >> 5];
        in.k[p] = load_f32(Kp, c);
        in.held[p] = load_f32(Hprev, c);
    }
}

template <typename T>
__device__ __forceinline__ void finish_column(const ColumnIn &in, EntryChunk *__restrict__ ents0,
                                              uint32_t *__restrict__ counts0, uint8_t *__restrict__ nch0,
                                              uint32_t *blk_cnt, int n, int d, int lane, int j, int slot_in_block) {
    if (j >= n) {
        if (lane == 0) blk_cnt[slot_in_block] = 0u;
        return;
    }
    const size_t row = (size_t)j;
    EntryChunk *out = ents0 + row * (d / kGroup);
    uint32_t off = 0;
    bool big = false;
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
        if (p * kWave >= d) break;
        const int c = p * kWave + lane;
        const bool act = c < d;
        bool bit = false;
        float delta = 0.f;
        if (act) {
            bit = (in.word[p] >> (c & 31)) & 1u;
            const float k = in.k[p];
            const float held = (j == 0) ? 0.f : in.held[p];
            delta = k - held;                                  // (row 0: the basis, delta = k)
            const float now = (bit || j == 0) ? k : held;      // reference key after this row
            big = big || !(fabsf(now) < 32768.f);
        }
        big = __any(big);
        const uint64_t b = __ballot(bit);
        if (bit) {
            const uint32_t slot = off + lanes_below(b);
            out[slot / kGroup].chan[slot % kGroup] = (uint32_t)c;
            out[slot / kGroup].delta[slot % kGroup] = delta;
        }
        off += __popcll(b);
    }
    uint32_t padded = (off + kGroup - 1) & ~(uint32_t)(kGroup - 1);
    if (padded == 0) padded = kGroup;
    if (off + lane < padded) {
        const uint32_t slot = off + lane;
        out[slot / kGroup].chan[slot % kGroup] = 0u;
        out[slot / kGroup].delta[slot % kGroup] = 0.f;
    }
    if (lane == 0) {
        counts0[row] = off;
        nch0[j] = (uint8_t)(padded / kGroup);
        // bit 31: some reference key of this row is too large for (or not a number in) fp16, the format in which the
        // matrix-core prefill kernel re-bases a column; such a column is gathered like any other
        blk_cnt[slot_in_block] = (padded / kGroup) | (big ? 0x80000000u : 0u);
    }
}

// Columns first, first + step, ... below end (end - first a multiple of step is not required) by one wave, the
// inputs of column i + 1 requested before column i is compacted; the chunk count of column j goes to
// blk_cnt[j - cnt_base].
template <typename T>
__device__ __forceinline__ void emit_columns(const T *K0, const T *H0, const uint32_t *M0, EntryChunk *__restrict__ ents0,
                                             uint32_t *__restrict__ counts0, uint8_t *__restrict__ nch0,
                                             uint32_t *blk_cnt, int n, int d, int lane, int first, int step, int end,
                                             int cnt_base) {
    if (first >= end) return;
    ColumnIn cur, nxt;
    load_column(cur, K0, H0, M0, n, d, lane, first);
    for (int j = first; j < end; j += step) {
        load_column(nxt, K0, H0, M0, n, d, lane, j + step);   // clamped to the last row; unused after the last column
        finish_column<T>(cur, ents0, counts0, nch0, blk_cnt, n, d, lane, j, j - cnt_base);
        cur = nxt;
    }
}

// The gather plan of one block of 32 key columns (see emit_entries_kernel), by the 64 lanes of one wave.
//   blk_cnt  [32] chunk counts of the block's columns (bit 31: a reference key of that row does not fit fp16)
//   plan_out the block's kPlanWaveCount x 8 bytes;  dense_out the block's word of re-based columns
constexpr int kPlanCols = 32, kPlanWaveCount = 8;            // columns per block = the prefill kernel's key block
constexpr int kRouteMin = 4;
__device__ __forceinline__ void plan_block(const uint32_t *blk_cnt, uint8_t *plan_out, uint32_t *dense_out, bool whole,
                                           int d, int lane) {
    constexpr int kCols = kPlanCols, kPlanWaves = kPlanWaveCount;
    const int c = lane & (kCols - 1);
    auto chunks_of = [&](int col) { return blk_cnt[col] & 0x7fffffffu; };
    const uint64_t full_cols = __ballot(lane < kCols && chunks_of(c) == (uint32_t)(d / kGroup));
    const bool fits = whole && !__any((blk_cnt[c] >> 31) != 0u) && __popcll(full_cols) >= kRouteMin;
    auto is_routed = [&](int col) { return fits && chunks_of(col) == (uint32_t)(d / kGroup); };
    const bool routed = is_routed(c);
    const uint64_t routed_cols = __ballot(routed && lane < kCols);
    const uint32_t mine = routed ? 0u : chunks_of(c);
    uint32_t rank = 0;
    for (int o = 0; o < kCols; ++o) {
        const uint32_t other = is_routed(o) ? 0u : chunks_of(o);
        rank += (other > mine || (other == mine && o < c)) ? 1u : 0u;
    }
    if (!whole) rank = (uint32_t)c;
    const uint32_t pair = rank >> 1;
    // The pairs go, longest first, to the wave whose SIMD has the fewest gather steps so far (waves w and w + 4 of the
    // 8 share a SIMD and its vector ALU; ties: the wave with fewer steps, then the lower index), two pairs per wave.
    // A whole-vector jump of the key stream - a column of d / 8 chunks among columns a third as long - then lands on a
    // SIMD whose other pairs are short.  (Dealt by rank alone, pairs w and 15 - w to wave w: 8.25 instead of 8.09 ms on
    // the 8K workload; treating waves w and w ^ 1 as SIMD partners instead: 8.38 ms.)
    // (lane w < 8 keeps wave w's tally; the choice is a minimum over those 8 lanes)
    uint32_t steps_mine = 0, pairs_mine = 0;                 // of wave `lane & 7`
    uint32_t wv = 0, nth = 0;                                // this lane's column: its wave, first or second pair there
    for (int r = 0; r < kCols / 2; ++r) {
        // steps of pair r = chunk count of its longer column, the one of rank 2 r
        const uint64_t holder = __ballot(lane < kCols && rank == (uint32_t)(2 * r));
        const uint32_t a = (uint32_t)__shfl((int)mine, (int)__builtin_ctzll(holder | (1ull << 63)));
        const uint32_t partner = (uint32_t)__shfl_xor((int)steps_mine, kPlanWaves / 2);
        uint32_t key = pairs_mine < 2u ? ((steps_mine + partner) << 16) | (steps_mine << 4) | (uint32_t)(lane & (kPlanWaves - 1))
                                       : 0xffffffffu;
#pragma unroll
        for (int sft = 1; sft < kPlanWaves; sft <<= 1) key = min(key, (uint32_t)__shfl_xor((int)key, sft));
        const uint32_t best = key & (uint32_t)(kPlanWaves - 1);
        const uint32_t had = (uint32_t)__shfl((int)pairs_mine, (int)best);
        if (pair == (uint32_t)r) {
            wv = best;
            nth = had;
        }
        if ((uint32_t)(lane & (kPlanWaves - 1)) == best) {
            steps_mine += a;
            pairs_mine += 1u;
        }
    }
    const uint32_t slot = 2u * nth + (rank & 1u);
    if (lane < kCols) {
        uint8_t *out = plan_out + wv * 8;
        out[slot] = (uint8_t)c;
        out[4 + slot] = whole ? (uint8_t)mine : (uint8_t)0;
    }
    if (lane == 0) *dense_out = (uint32_t)routed_cols;
}

}  // namespace da
