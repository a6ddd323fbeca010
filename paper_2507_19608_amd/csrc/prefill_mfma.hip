// Hybrid-attention prefill for bf16 inputs, head_dim 64 or 128 (Sec. III-B prefill stage; Eq. 4; Eq. 1).
//
// Work group = 512 threads (8 waves) on 256 "score rows": RT consecutive query rows x GH query heads of
// one KV head (they share K, V and the delta matrix).  Key columns are walked left to right in blocks
// of 32.  A row's window is its square of side W on the diagonal, or the band of the W newest keys.
//
//   far blocks   (every row of the tile has the column outside its window): Eq. 4 as written.  A wave
//                takes four columns of the block as two pairs of (nearly) equally long columns; its two halves
//                work on the two columns of a pair at once, a lane on 8 score rows, adding q[c] * delta for each
//                surviving (channel, delta) entry of its column.  The entry lists arrive as two-address LDS reads
//                from a per-wave ring; q comes from a transposed fp16 copy of the Q tile in LDS (one 16-byte read
//                feeds 8 multiply-adds).  The per-column updates u are exchanged through LDS; the owner of a score
//                row adds them up in column order (its running Eq. 4 score).  In blocks where the compaction kernel
//                has marked full columns for re-basing, the score at such a column is taken from a K_hat Q^T tile
//                on the matrix cores instead (Eq. 4 telescoped) and the running score continues from it.
//   near blocks  (some row has the column inside its window): exact scores K Q^T on the matrix cores;
//                where a tile straddles window squares, the not-yet-exact entries come from K_hat Q^T
//                (Eq. 4 telescoped: sum of the deltas up to column j is the held key k_hat(j)).
//   every block  online softmax with lane-local row state, P V on the matrix cores with V pre-transposed.
//
// Matrix-core layouts (v_mfma_f32_32x32x16_bf16, wave64): A lane l holds row l%32, k = 8*(l/32)..+7;
// B lane l holds column l%32, same k; D lane l holds column l%32, rows 8*(r/4) + 4*(l/32) + r%4 for
// register r.  Scores are produced transposed (keys x score rows) so that a lane owns one score row,
// and D registers 8a..8a+7 are exactly the B operand of the a-th k-step of P V once V^T is fetched in
// the matching key order.
#include "common.hpp"
#include "kernels.hpp"
#include "scan_device.hpp"
#include "vt_device.hpp"

namespace da {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) _Float16 half4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kRows = 256;      // score rows per work group
constexpr int kWaves = 8;

struct MfmaArgs {
    const bf16_t *__restrict__ Q;
    const bf16_t *__restrict__ K;
    const bf16_t *__restrict__ Khat;
    const bf16_t *__restrict__ Vt;      // per unit: V in matrix-core operand order, D * n_pad elements
    bf16_t *__restrict__ O;
    const EntryChunk *__restrict__ ents;
    const uint8_t *__restrict__ plan;   // per unit and block of kTB columns: kWaves x 8 bytes (emit_entries_kernel)
    const uint32_t *__restrict__ dense; // per unit and block: bit c set = column c is re-based, not gathered
    int Hq, Hkv, n, n_pad, W, rebase, sliding;
    int ld, ld_pad;                     // rows of room per unit in K, Khat, V, ents, counts (>= n), and the padded
                                        // stride of Vt, nch8, plan, dense that goes with it (>= n_pad)
    int q_off, nq;                      // query rows are positions q_off .. q_off + nq - 1 of the n keys
    int GH, RT, tiles, hgroups;         // heads per group chunk, rows per tile, row tiles, head chunks per unit
    int xsplit;                         // > 0: XCD-aware order, every unit split this many ways (see the kernel)
    int ksplit;                         // >= 1: most work groups a tile gets, each on a part of the tile's key blocks
    int parts_total;                    // sum over a unit's row tiles of TileGeometry::parts (= tiles when ksplit == 1)
    float *__restrict__ part_o;         // ksplit > 1: [tile][ksplit][256][D] unnormalised outputs of the parts
    float *__restrict__ part_ml;        //             [tile][ksplit][256][2] their running maximum and sum
    float scale_log2;
    // fused short-prompt launch only: what the stand-alone scan, compaction and V re-order kernels take
    const bf16_t *__restrict__ V;       // [unit][n][D] as the caller passed it
    uint32_t *__restrict__ mask_bits;   // out
    unsigned long long *__restrict__ nnz;   // out
    uint32_t *__restrict__ counts;
    uint8_t *__restrict__ nch8;
    float theta;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;

template <int D>
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16_t *__restrict__ V, bf16_t *__restrict__ Vt,
                                                          int n, int ld, int ld_pad, int blk0) {
    __shared__ bf16_t tile[kTB][D + 2];
    constexpr int MT = D / 32;
    const int unit = blockIdx.y, blk = blk0 + blockIdx.x;
    transpose_v_block<D, 256>(V + (size_t)unit * ld * D,
                              (u32x4 *)(Vt + (size_t)unit * D * ld_pad) + (size_t)blk * (2 * MT * 64), blk * kTB, n, tile,
                              (int)threadIdx.x, [] { __syncthreads(); });
}

// A tile (kRows score rows: RT query rows from position i0 on, of GH heads) and how its key blocks are split.
// Key blocks 0 .. far_blocks - 1 lie left of every row's window (gather mode only: they take the Eq. 4 gather), the
// rest up to nblocks go through the matrix cores.  A launch may give every tile `ksplit` work groups ("parts"), each
// on a contiguous range of the tile's blocks, whose unnormalised outputs a second launch merges (flash-decoding
// style); that is done when a gather-mode launch has too few tiles to fill the chip.  A tile is cut into at most one
// part per kSplitMinBlocks gather blocks, so short tiles are not cut at all and write their output themselves.  A
// gather part that does not start at block 0 starts its running score from the dense product q . k_hat(j - 1) of the
// column before its first (Eq. 4 telescoped).
constexpr int kSplitMinBlocks = 4;   // (measured 2 .. 8 on prompts of 512 .. 4096 tokens: 4 is best or level everywhere)
struct TileGeometry {
    int i0, i_last;        // first and last query position
    int win_first;         // smallest window start of the tile's rows
    int far_blocks, nblocks;
    int parts;             // work groups that share the tile (<= ksplit)
};
// (host and device: the launcher sizes the grid by the sum of `parts` over the tiles)
__host__ __device__ inline TileGeometry tile_geometry_of(int q_off, int RT, int n, int W, int sliding, int ksplit,
                                                         bool gather, int tile) {
    TileGeometry g;
    g.i0 = q_off + tile * RT;
    g.i_last = g.i0 + RT - 1 < n - 1 ? g.i0 + RT - 1 : n - 1;
    g.win_first = sliding ? (g.i0 - W + 1 > 0 ? g.i0 - W + 1 : 0) : (g.i0 / W) * W;
    g.far_blocks = gather ? g.win_first / kTB : 0;
    g.nblocks = g.i_last / kTB + 1;
    const int cut = (gather ? g.far_blocks : g.nblocks) / kSplitMinBlocks;   // (rounded down: up or to nearest measured worse)
    g.parts = cut < 1 ? 1 : (cut < ksplit ? cut : ksplit);
    return g;
}
template <bool kGather>
__device__ __forceinline__ TileGeometry tile_geometry(const MfmaArgs &a, int tile) {
    return tile_geometry_of(a.q_off, a.RT, a.n, a.W, a.sliding, a.ksplit, kGather, tile);
}
// blocks [lo, hi) of `count` blocks that part `seg` of `parts` takes
__device__ __forceinline__ int part_begin(int count, int seg, int parts) { return (int)((long long)count * seg / parts); }

// What the stand-alone scan, compaction and V re-order launches do for a unit, done by one work group of the fused
// short-prompt kernel for the key rows 0 .. need - 1 that its own query rows see (512 threads; `lds` is scratch of
// fused_lds_bytes(D, need) bytes that nothing else uses yet).  The key rows are copied into LDS once; Eq. 2-3 run
// there row by row (wave ballot = mask word), leaving the reference keys and mask words beside them in LDS; the
// compaction (ballot + prefix count per column) reads all three from LDS and writes the entry lists and gather plans
// to the workspace, from where the gather loop streams them into its rings as in the multi-launch path.
// Every work group of a unit does this on its own and writes the same workspace arrays with the same values (only
// final values are ever stored, and only for rows and blocks all of whose inputs the work group holds): a work group
// reads only what it has itself written, whatever the others are doing.
// `writer` (one work group per unit, one that needs every row) also stores the unit's nnz.
__host__ __device__ constexpr size_t fused_lds_bytes(int d, int need) {
    return 64 + (size_t)2 * need * d * 2 + (size_t)need * (d / 32) * 4 + (size_t)need * 4;
}

template <int D>
__device__ __forceinline__ void fused_prepare(const MfmaArgs &a, int unit, int need, int gather_blocks, bool writer,
                                              char *lds) {
    constexpr int CW = D / kWave;                               // waves that scan (64 channels each)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = a.n;
    const bf16_t *Kp = a.K + (size_t)unit * a.ld * D;
    bf16_t *Hp = const_cast<bf16_t *>(a.Khat) + (size_t)unit * a.ld * D;
    uint32_t *Mp = a.mask_bits + (size_t)unit * n * (D / 32);
    unsigned long long *cnt = (unsigned long long *)lds;        // [CW] surviving entries per scanning wave
    bf16_t *Kl = (bf16_t *)(lds + 64);                          // [need][D] keys
    bf16_t *Hl = Kl + (size_t)need * D;                         // [need][D] reference keys
    uint32_t *Ml = (uint32_t *)(Hl + (size_t)need * D);         // [need][D / 32] mask words
    // 1. the key rows into LDS
    {
        constexpr int kPer = kFusedMaxElems / 8 / 512;           // 16-byte pieces per thread at the largest prompt
        u32x4 piece[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {                         // every load issued before the first is parked
            const int idx = tid + i * 512;
            piece[i] = ((const u32x4 *)Kp)[min(idx, need * (D / 8) - 1)];
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int idx = tid + i * 512;
            if (idx < need * (D / 8)) ((u32x4 *)Kl)[idx] = piece[i];
        }
    }
    __syncthreads();
    // 2. Eq. 2-3 over the rows, in order, by CW waves (64 channels each)
    if (wave < CW) {
        unsigned long long c = 0;
        scan_rows<bf16_t, true>(Kl, Hl, Ml, D, wave * kWave + lane, lane, 0, need, true, (const bf16_t *)nullptr, 0.f,
                                a.theta, &c);
        if (lane == 0) cnt[wave] = c;
    }
    __syncthreads();
    // 3. reference keys and mask words out to the workspace / the caller's mask array; nnz
    for (int idx = tid; idx < need * (D / 8); idx += 512) ((u32x4 *)Hp)[idx] = ((const u32x4 *)Hl)[idx];
    for (int idx = tid; idx < need * (D / 32); idx += 512) Mp[idx] = Ml[idx];
    if (writer && tid == 0) {
        unsigned long long t = 0;
        for (int w = 0; w < CW; ++w) t += cnt[w];
        a.nnz[unit] = t;
    }
    // 4. compaction of the key columns of the blocks this work group will gather (whole blocks left of every one of
    //    its rows' windows, so all their rows are here), a column per wave at a time, then their gather plans
    uint32_t *blk_cnt = (uint32_t *)(Ml + (size_t)need * (D / 32));   // [gather_blocks][32] chunk counts
    EntryChunk *ents0 = const_cast<EntryChunk *>(a.ents) + (size_t)unit * a.ld * (D / kGroup);
    uint32_t *counts0 = a.counts + (size_t)unit * a.ld;
    uint8_t *nch0 = a.nch8 + (size_t)unit * a.ld_pad;
    uint8_t *plan = const_cast<uint8_t *>(a.plan) + (size_t)unit * (a.ld_pad / kTB) * kWaves * 8;
    uint32_t *dense = const_cast<uint32_t *>(a.dense) + (size_t)unit * (a.ld_pad / kTB);
    emit_columns((const bf16_t *)Kl, (const bf16_t *)Hl, (const uint32_t *)Ml, ents0, counts0, nch0, blk_cnt, need, D,
                 lane, wave, kWaves, gather_blocks * kTB, 0);
    lds_barrier();                                               // (the chunk counts; the lists go to global memory)
    for (int blk = wave; blk < gather_blocks; blk += kWaves)
        plan_block(blk_cnt + blk * kTB, plan + (size_t)blk * kWaves * 8, dense + blk, (blk + 1) * kTB <= n, D, lane);
    __syncthreads();
    // 5. V into matrix-core operand order, a block of 32 keys per wave at a time (the LDS copies above are done with)
    {
        typedef bf16_t (*tile_t)[D + 2];
        tile_t tile = (tile_t)(lds + 64 + (size_t)wave * kTB * (D + 2) * sizeof(bf16_t));
        const bf16_t *Vp = a.V + (size_t)unit * a.ld * D;
        u32x4 *Op = (u32x4 *)(const_cast<bf16_t *>(a.Vt) + (size_t)unit * D * a.ld_pad);
        for (int blk = wave; blk * kTB < need; blk += kWaves)
            transpose_v_block<D, kWave>(Vp, Op + (size_t)blk * (2 * (D / 32) * 64), blk * kTB, n, tile, lane, [] {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            });
    }
    __threadfence();
    __syncthreads();
}

// kGather: Eq. 4 as written for the far blocks (DA_SCORE_GATHER); otherwise every block goes through the matrix
// cores (DA_SCORE_REBASE) and neither the fp16 Q tile nor the gather loop exists in the instantiation.
// kAligned: the launcher has checked that every tile's rows share one window whose start is a multiple of the block
// size; the K_hat tile of the near blocks, its loads and its branches then do not exist in the instantiation.
// kFused: the work group first runs the delta scan, the compaction and the V re-order for its unit itself (short
// prompts: one launch instead of seven; see fused_prepare), and reads its gather plans with vector loads.
template <int D, bool kGather, bool kAligned, bool kFused = false>
__global__ __launch_bounds__(512) void prefill_mfma_kernel(MfmaArgs a) {
    // (aligned explicitly: the dynamic region starts where the static variables below end, and every tile and ring
    // in it is accessed with 16-byte instructions - at an offset that was not a multiple of 16 the far loop ran seven
    // times slower)
    extern __shared__ __attribute__((aligned(256))) char lds_raw[];
    constexpr size_t kQtBytes = kGather ? (size_t)D * kRows * 2 : 0;
    _Float16 *qt = (_Float16 *)lds_raw;                                   // [D][256] fp16, scaled by 2^qexp
    float *ubuf = (float *)(lds_raw + kQtBytes);                          // [kTB][256]; then 8 entry rings
    __shared__ float red[kWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction; tell the compiler
    const int half = lane >> 5, li = lane & 31;

    // ---- which tile.  Work groups go to the 8 XCDs round-robin by index, and every XCD has its own L2; all
    //      tiles of a unit stream the same K, K_hat, V and entry lists.  So the index is first turned into
    //      (XCD, slot on that XCD), and each XCD is given whole units - or, when the unit count does not
    //      divide by 8, units split `xsplit` ways by tile index modulo xsplit - one after the other: a unit's
    //      streams are then fetched into xsplit L2s instead of all 8.  Within a part, heavy (late) tiles first.
    int bid = blockIdx.x;
    const int per_unit = a.parts_total * a.hgroups;
    if (a.xsplit > 0) {
        const int xcd = bid & 7, slot = bid >> 3;
        const int per_part = per_unit / a.xsplit;            // work groups of one part
        const int part = xcd + 8 * (slot / per_part);        // parts xcd, xcd + 8, ... belong to this XCD
        const int within = slot % per_part;
        bid = (part / a.xsplit) * per_unit + within * a.xsplit + part % a.xsplit;
    }
    // Without the XCD-aware order, a launch that is cut along the keys (few, long tiles) deals its work groups out
    // heaviest first across all units - unit after unit, the heavy tiles of the last unit would start last; an uncut
    // launch goes unit after unit, so that all its work groups stream the same unit's tiles at a time.
    const int units = gridDim.x / per_unit;
    const bool across = a.xsplit == 0 && a.ksplit > 1;
    const int unit = across ? bid % units : bid / per_unit;
    bid = across ? bid / units : bid - unit * per_unit;
    const int hchunk = bid % a.hgroups;
    // The unit's parts are numbered tile by tile from the last (heaviest) tile down, a tile's parts in a row: every
    // index of the grid is a part that exists (work groups that only find out that they have nothing to do still
    // hold up the ones queued behind them when a launch has more of them than the chip has room for).
    int tile = a.tiles - 1 - bid / a.hgroups, seg = 0;
    if (a.ksplit > 1) {
        int q = bid / a.hgroups;
        for (tile = a.tiles - 1; tile > 0; --tile) {
            const int p = tile_geometry<kGather>(a, tile).parts;
            if (q < p) break;
            q -= p;
        }
        seg = q;
    }
    const int b = unit / a.Hkv, hk = unit % a.Hkv;
    const int g = a.Hq / a.Hkv;
    const int head0 = hk * g + hchunk * a.GH;
    const int n = a.n, W = a.W, RT = a.RT;
    const TileGeometry geo = tile_geometry<kGather>(a, tile);
    const int i0 = geo.i0, i_last = geo.i_last;
    if (seg >= geo.parts) return;                            // a short tile is not split as many ways as the launch allows

    const bf16_t *Kp = a.K + (size_t)unit * a.ld * D;
    const bf16_t *Hp = a.Khat + (size_t)unit * a.ld * D;
    const bf16_t *Vtp = a.Vt + (size_t)unit * D * a.ld_pad;
    const EntryChunk *Ep = a.ents + (size_t)unit * a.ld * (D / kGroup);
    const uint8_t *Pp = a.plan + (size_t)unit * (a.ld_pad / kTB) * (kWaves * 8);
    const uint32_t *Dp = a.dense + (size_t)unit * (a.ld_pad / kTB);

    // score row sr = hh * RT + r  ->  query row i0 + r of head head0 + hh
    auto q_row_ptr = [&](int sr) -> const bf16_t * {
        const int hh = sr / RT, r = sr - hh * RT;
        const int i = min(i0 + r, n - 1);
        return a.Q + (((size_t)b * a.Hq + head0 + hh) * a.nq + (i - a.q_off)) * D;
    };

    if constexpr (kFused) {
        const int first_win = a.sliding ? max(i0 - W + 1, 0) : (i0 / W) * W;   // window start of the tile's first row
        fused_prepare<D>(a, unit, min(n, i_last + 1), kGather ? first_win / kTB : 0, tile == a.tiles - 1 && hchunk == 0,
                         lds_raw);
    }

    float qmul = 1.f;
    if constexpr (kGather) {
        // ---- stage the Q tile: per-tile power-of-two scale so that the fp16 copy neither overflows nor
        //      loses bits that matter (|q| max lands in [2^14, 2^15)).
        //      The tile is read once: a thread keeps its pieces (score row idx % 256, 8 channels) in registers from
        //      the pass that finds the maximum to the pass that scales and stores them.
        constexpr int kQPer = kRows * (D / 8) / 512;             // 16-byte pieces per thread
        u32x4 raw[kQPer];
        float amax = 0.f;
#pragma unroll
        for (int p = 0; p < kQPer; ++p) {
            const int idx = tid + p * 512, sr = idx % kRows, c8 = idx / kRows;   // consecutive threads -> consecutive score rows
            raw[p] = *(const u32x4 *)(q_row_ptr(sr) + c8 * 8);
        }
#pragma unroll
        for (int p = 0; p < kQPer; ++p)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                amax = fmaxf(amax, fabsf(__uint_as_float(raw[p][k] << 16)));
                amax = fmaxf(amax, fabsf(__uint_as_float(raw[p][k] & 0xffff0000u)));
            }
    #pragma unroll
        for (int s = 32; s >= 1; s >>= 1) amax = fmaxf(amax, __shfl_xor(amax, s));
        if (lane == 0) red[wave] = amax;
        __syncthreads();
        amax = red[0];
    #pragma unroll
        for (int k = 1; k < kWaves; ++k) amax = fmaxf(amax, red[k]);
        int qexp = 0;
        if (amax > 0.f && amax < INFINITY) {
            const int e = (int)((__float_as_uint(amax) >> 23) & 0xff) - 127;   // floor(log2 amax) for normal values
            qexp = 14 - e;
        }
        qmul = __uint_as_float((uint32_t)(min(max(qexp, -126), 127) + 127) << 23);
#pragma unroll
        for (int p = 0; p < kQPer; ++p) {
            const int idx = tid + p * 512, sr = idx % kRows, c8 = idx / kRows;
    #pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float lo = __uint_as_float(raw[p][k] << 16) * qmul;
                const float hi = __uint_as_float(raw[p][k] & 0xffff0000u) * qmul;
                qt[(c8 * 8 + 2 * k) * kRows + sr] = (_Float16)lo;
                qt[(c8 * 8 + 2 * k + 1) * kRows + sr] = (_Float16)hi;
            }
        }
    }
    const float far_scale = a.scale_log2 / qmul;   // undo the tile scale together with the softmax scale

    // ---- this wave's score rows for softmax / PV: sr = 32 * wave + li (both lane halves)
    const int my_sr = 32 * wave + li;
    const int my_hh = my_sr / RT, my_r = my_sr - my_hh * RT;
    const int my_i = i0 + my_r;
    const bool my_valid = my_i < n;
    // first exact column of row r: start of its square, or of its band (monotone in r either way)
    auto win_start = [&](int r) { return a.sliding ? max(r - W + 1, 0) : (r / W) * W; };
    const int my_win = win_start(min(my_i, n - 1));
    const bf16_t *my_q = q_row_ptr(my_sr);

    constexpr int KS = D / 16;     // k-steps of Q K^T
    constexpr int MT = D / 32;     // channel tiles of the output

    f32x16 oacc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[mt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    // Eq. 4 running score of this lane's score row at the end of the previous block.  Inside a block the column updates
    // are added up in binary32; across blocks the total is kept in binary64 (one add per block), so that the rounding
    // of the one long sum does not grow with the prompt length (in binary32 it showed at ~130 000 columns).
    double r_run = 0.0;

    const int win_first = geo.win_first;         // smallest window start of the tile's rows
    const int win_last = win_start(i_last);      // largest
    const bool aligned = kAligned || ((win_first % kTB == 0) && (win_first == win_last));
    const int far_blocks = geo.far_blocks;
    const int nblocks = geo.nblocks;
    // this work group's part of the tile: gather blocks [f_lo, f_hi), matrix-core blocks [n_lo, n_hi)
    const int f_lo = kGather ? part_begin(far_blocks, seg, geo.parts) : 0;
    const int f_hi = kGather ? part_begin(far_blocks, seg + 1, geo.parts) : 0;
    const int n_lo = kGather ? (seg == geo.parts - 1 ? far_blocks : nblocks) : part_begin(nblocks, seg, geo.parts);
    const int n_hi = kGather ? nblocks : part_begin(nblocks, seg + 1, geo.parts);
    if (kGather && f_lo > 0) {
        // running score at the end of column 32 f_lo - 1, in the units of the gather (the Q tile's scale): bf16
        // products are exact in binary32, the sum is taken in binary64
        const bf16_t *hrow = Hp + (size_t)(f_lo * kTB - 1) * D;
        double acc = 0.0;
        u32x4 qrow[D / 8];                                        // (all of the row's loads in flight at once)
#pragma unroll
        for (int c8 = 0; c8 < D / 8; ++c8) qrow[c8] = *(const u32x4 *)(my_q + c8 * 8);
#pragma unroll
        for (int c8 = 0; c8 < D / 8; ++c8) {
            const u32x4 qv = qrow[c8], hv = *(const u32x4 *)(hrow + c8 * 8);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                acc += (double)(__uint_as_float(qv[k] << 16) * __uint_as_float(hv[k] << 16));
                acc += (double)(__uint_as_float(qv[k] & 0xffff0000u) * __uint_as_float(hv[k] & 0xffff0000u));
            }
        }
        r_run = acc * (double)qmul;
    }

    __syncthreads();   // Q tile staged

    // V^T operands of one block: vreg[ka * MT + mt] for k-step ka, channel tile mt.  V was rearranged
    // into matrix-core operand order, so each operand is one fully coalesced 16-byte load per lane.
    auto load_v = [&](u32x4 (&vreg)[2 * MT], int jb) {
        const u32x4 *vp = (const u32x4 *)Vtp + (size_t)(jb / kTB) * (2 * MT * 64) + lane;
#pragma unroll
        for (int k = 0; k < 2 * MT; ++k) vreg[k] = vp[k * 64];
    };

    // Online softmax + PV for one block; s[16] are this lane's raw scores (-inf where masked), sc the
    // positive factor that turns them into log2 units.  The running maximum is only raised when the
    // block maximum exceeds it by more than 2^8 in the exponent, so probabilities stay <= 256 and the
    // accumulator is rarely rescaled.
    auto softmax_pv = [&](float (&s)[16], float sc, const u32x4 (&vreg)[2 * MT]) {
        float bm = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) bm = fmaxf(bm, s[r]);
        bm = fmaxf(bm, __shfl_xor(bm, 32)) * sc;
        if (__any(bm > m_run + 8.f)) {
            const float m_new = fmaxf(m_run, bm);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[mt][r] *= alpha;
        }
        const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
            p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], sc, neg_m));   // bare v_exp_f32: tiny results may flush to 0
        // The row sum is taken over the probabilities as rounded to bf16, i.e. over the very weights that P V uses:
        // the output is then an exact weighted mean of the value rows, and the rounding of the weights cannot bias it
        // (summing the unrounded ones does, by up to 2^-9 relative when many weights are equal).
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        float psum = 0.f;
#pragma unroll
        for (int ka = 0; ka < 2; ++ka) {
            u32x4 pb;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                f32x2 pr;
                pr[0] = p[8 * ka + 2 * k];
                pr[1] = p[8 * ka + 2 * k + 1];
                const bf16x2 pk = __builtin_convertvector(pr, bf16x2);
                psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);
                pb[k] = __builtin_bit_cast(uint32_t, pk);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vreg[ka * MT + mt]), as_bf16x8(pb),
                                                                  oacc[mt], 0, 0, 0);
        }
        l_run += psum;
    };

    // ---------------------------------------------------------------- far blocks: gather (Eq. 4)
    // A wave takes four columns of every block, as two pairs of columns with (nearly) equal numbers of entry
    // chunks, dealt out beforehand (emit_entries_kernel).  The entry chunks of those columns travel
    // global memory -> registers (one 16-byte load per lane, a whole block ahead) -> a private LDS
    // ring where the block's chunks sit back to back.  The two halves of the wave then work on the two columns of
    // a pair at the same time, a lane on 8 score rows: one two-address 16-byte LDS read fetches a piece of a chunk
    // of either column, one 16-byte q read per entry feeds 8 multiply-adds.  No scalar memory load sits in the
    // inner loop, so all its LDS traffic completes in order; the loop is software-pipelined two chunks deep.
    if (kGather && f_lo < f_hi) {
        const char *qtb = (const char *)qt;
        constexpr int kRingBytes = 4 * (D / kGroup) * 64 + 4 * 64;
        char *ring = lds_raw + kQtBytes + (size_t)kTB * kRows * 4 + (size_t)wave * kRingBytes;
        for (int o = lane * 16; o < kRingBytes; o += 64 * 16) *(u32x4 *)(ring + o) = u32x4{0u, 0u, 0u, 0u};

        // this wave's columns of a block: .x = their indices inside the block, .y = their chunk counts, one byte each;
        // bytes 0, 1 are the first pair (longer column first), bytes 2, 3 the second
        // .z = the block's re-based columns (the same word for every wave)
        typedef __attribute__((ext_vector_type(3))) uint32_t u32x3;
        auto pack_of = [&](int blk) -> u32x3 {
            if (blk >= f_hi) return u32x3{0u, 0u, 0u};
            if constexpr (kFused) {
                // written earlier by this very work group with vector stores: read back through the same (vector)
                // cache, which sees them; the scalar cache need not
                const uint32_t *pp = (const uint32_t *)(Pp + ((size_t)blk * kWaves + wave) * 8);
                const uint32_t x = __builtin_nontemporal_load(pp), y = __builtin_nontemporal_load(pp + 1);
                const uint32_t z = __builtin_nontemporal_load(Dp + blk);
                return u32x3{(uint32_t)__builtin_amdgcn_readfirstlane((int)x), (uint32_t)__builtin_amdgcn_readfirstlane((int)y),
                             (uint32_t)__builtin_amdgcn_readfirstlane((int)z)};
            } else {
                const const_u32_ptr pp = (const_u32_ptr)(uintptr_t)(Pp + ((size_t)blk * kWaves + wave) * 8);
                const const_u32_ptr dp = (const_u32_ptr)(uintptr_t)(Dp + blk);
                return u32x3{pp[0], pp[1], dp[0]};
            }
        };
        auto g_issue = [&](u32x4 (&st)[4], int blk, u32x3 pk) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const uint32_t nch = (pk[1] >> (8 * cc)) & 0xffu, col = (pk[0] >> (8 * cc)) & 0xffu;
                st[cc] = u32x4{0u, 0u, 0u, 0u};
                if ((uint32_t)lane < 4u * nch)
                    st[cc] = *(const u32x4 *)((const char *)(Ep + (size_t)(blk * kTB + col) * (D / kGroup)) + lane * 16);
            }
        };
        auto w_store = [&](const u32x4 (&st)[4], u32x3 pk) {
            uint32_t base = 0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const uint32_t nch = (pk[1] >> (8 * cc)) & 0xffu;
                if ((uint32_t)lane < 4u * nch) *(u32x4 *)(ring + base * 64 + lane * 16) = st[cc];
                base += nch;
            }
        };

        typedef __attribute__((ext_vector_type(8))) _Float16 half8;
        typedef const half8 __attribute__((address_space(3))) *lds_half8_ptr;
        typedef const u32x4 __attribute__((address_space(3))) *lds_u32x4_ptr;
        typedef const f32x4 __attribute__((address_space(3))) *lds_f32x4_ptr;
        struct Set {
            half8 q[8];     // q values of 8 score rows at the chunk's 8 channels
            f32x4 d[2];     // the chunk's 8 deltas
        };
        constexpr uint32_t kZeroChunk = 4 * (D / kGroup);       // first chunk of the ring's zero pad, never written
        const uint32_t ring_lds = (uint32_t)(uintptr_t)(char __attribute__((address_space(3))) *)ring;
        const uint32_t q_lane = (uint32_t)(uintptr_t)(const char __attribute__((address_space(3))) *)qtb +
                                (uint32_t)(lane & 31) * 16u;
        const uint32_t zero_addr = ring_lds + kZeroChunk * 64u;

        u32x3 pk_cur = pack_of(f_lo), pk_nxt = pack_of(f_lo + 1);
        u32x4 st[4];
        g_issue(st, f_lo, pk_cur);

        auto gather_block = [&](u32x3 pk) {
            uint32_t first = 0;                                  // first ring chunk of the pair's longer column
#pragma unroll
            for (int pair = 0; pair < 2; ++pair) {
                const uint32_t na = (pk[1] >> (16 * pair)) & 0xffu, nb = (pk[1] >> (16 * pair + 8)) & 0xffu;
                const uint32_t ca = (pk[0] >> (16 * pair)) & 0xffu, cb = (pk[0] >> (16 * pair + 8)) & 0xffu;
                const uint32_t steps = na;                       // na >= nb
                const uint32_t my_n = half ? nb : na, my_col = half ? cb : ca;
                const uint32_t my_first = ring_lds + (half ? first + na : first) * 64u;
                first += na + nb;
                auto chunk_addr = [&](uint32_t t) { return t < my_n ? my_first + t * 64u : zero_addr; };
                float u[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) u[r] = 0.f;
                if (steps > 0) {                                 // (a pair of re-based columns has nothing to gather)
                Set S0, S1;
                u32x4 chn[2];                                    // channel indices of the chunk whose q reads come next
                auto rd_ch = [&](uint32_t a) {
                    chn[0] = *(lds_u32x4_ptr)(uintptr_t)(a);
                    chn[1] = *(lds_u32x4_ptr)(uintptr_t)(a + 16u);
                };
                auto rd_d = [&](Set &x, uint32_t a) {
                    x.d[0] = *(lds_f32x4_ptr)(uintptr_t)(a + 32u);
                    x.d[1] = *(lds_f32x4_ptr)(uintptr_t)(a + 48u);
                };
                auto issue_q = [&](Set &x) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        x.q[i] = *(lds_half8_ptr)(uintptr_t)(chn[i >> 2][i & 3] * (uint32_t)(kRows * 2) + q_lane);
                };
                uint32_t a_next = chunk_addr(0);
                rd_ch(a_next);
                issue_q(S0);
                rd_d(S0, a_next);
                a_next = chunk_addr(1);
                rd_ch(a_next);
                // consume chunk t (set x) while the q / delta reads of chunk t+1 (set y, issued here) and the channel
                // reads of chunk t+2 are in flight
                auto step = [&](Set &x, Set &y, uint32_t t) {
                    issue_q(y);
                    rd_d(y, a_next);
                    a_next = chunk_addr(t + 2);
                    rd_ch(a_next);
                    // keep the reads above ahead of the multiply-adds below: left alone, the compiler at times sinks
                    // each q read to just before its use (one register quad, a full LDS wait per entry)
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float dl = x.d[i >> 2][i & 3];
#pragma unroll
                        for (int r = 0; r < 8; ++r) u[r] = fmaf((float)x.q[i][r], dl, u[r]);
                    }
                };
                uint32_t t = 0;
                for (; t + 1 < steps; t += 2) {
                    step(S0, S1, t);
                    step(S1, S0, t + 1);
                }
                if (t < steps) step(S0, S1, t);
                }
                // both columns of the pair are done: hand their update vectors to the score-row owners
                float *dst = ubuf + my_col * kRows + (lane & 31) * 8;
                *(f32x4 *)dst = f32x4{u[0], u[1], u[2], u[3]};
                *(f32x4 *)(dst + 4) = f32x4{u[4], u[5], u[6], u[7]};
            }
        };

        // K_hat Q^T tile of a block with re-based columns, on the matrix cores in fp16.  The K_hat rows of block b + 1 are
        // fetched once per work group (one 16-byte piece per thread, requested after the gather of block b), turned into
        // fp16 - exact: a bf16 value has 8 significant bits, and the compaction kernel routes a block's columns only if
        // its reference keys are below 2^15 - and parked in one of two LDS buffers in operand order at the end of
        // iteration b; the barrier of iteration b + 1 publishes them.  The query operand is read from the fp16 Q tile
        // the gather uses (8 two-byte reads per k-step: the tile is stored channel-major), so the product comes out in
        // the units of the running score and no operand is held in registers across the gather loop.
        constexpr int kHTileBytes = D * 64;                      // 32 keys x D channels, fp16
        constexpr int kHPieces = kHTileBytes / 16;
        char *hbuf = lds_raw + kQtBytes + (size_t)kTB * kRows * 4 + (size_t)kWaves * kRingBytes;
        const bool h_has_piece = kHPieces == 512 || tid < kHPieces;
        const int h_ptid = tid & (kHPieces - 1);
        const int h_pr = h_ptid & 31, h_pseg = h_ptid >> 5;      // key row of the block, 8-channel segment
        const int h_slot = ((h_pseg >> 1) * 64 + (h_pseg & 1) * 32 + h_pr) * 16;
        u32x4 hpiece;
        auto load_h_piece = [&](int blk) {
            hpiece = *(const u32x4 *)(Hp + (size_t)(blk * kTB + h_pr) * D + h_pseg * 8);
        };
        auto park_h_piece = [&](int blk) {
            u32x4 f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float lo = __uint_as_float(hpiece[k] << 16), hi = __uint_as_float(hpiece[k] & 0xffff0000u);
                f[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
            }
            if (h_has_piece) *(u32x4 *)(hbuf + (blk & 1) * kHTileBytes + h_slot) = f;
        };
        typedef __attribute__((ext_vector_type(8))) _Float16 half8v;
        auto rebase_tile = [&](int blk) -> f32x16 {
            f32x16 t0, t1;
#pragma unroll
            for (int r = 0; r < 16; ++r) t0[r] = t1[r] = 0.f;
            const char *ha = hbuf + (blk & 1) * kHTileBytes + lane * 16;
            const _Float16 *qb = qt + (size_t)(half * 8) * kRows + my_sr;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const half8v xa = __builtin_bit_cast(half8v, *(const u32x4 *)(ha + ks * 1024));
                half8v xq;
#pragma unroll
                for (int e = 0; e < 8; ++e) xq[e] = qb[(size_t)(ks * 16 + e) * kRows];
                if (ks & 1)
                    t1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa, xq, t1, 0, 0, 0);
                else
                    t0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa, xq, t0, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) t0[r] += t1[r];
            return t0;
        };
        // Scores of one block from its column updates uu (this lane's 16 columns, read from the exchange buffer), then
        // softmax and P V.  Keys of the block in groups of 4: group 2q belongs to lane half 0, group 2q+1 to half 1 (the
        // matrix-core D layout).  A lane sums inside its own groups and gets the other half's group totals from its
        // partner lane, so the running Eq. 4 score advances in column order.
        auto scores_softmax_pv = [&](int blk, const float (&uu)[16], uint32_t dm, const u32x4 (&vreg)[2 * MT]) {
            float s[16];
            if (dm == 0) {
                float w[16], t_own[4], t_oth[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float run = 0.f;
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        run += uu[4 * q + bb];
                        w[4 * q + bb] = run;
                    }
                    t_own[q] = run;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) t_oth[q] = __shfl_xor(t_own[q], 32);
                const float r0 = (float)r_run;
                float rel = 0.f;                                 // sum of this block's updates so far
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float mine = r0 + (half ? rel + t_oth[q] : rel);
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) s[4 * q + bb] = mine + w[4 * q + bb];
                    rel += t_own[q] + t_oth[q];
                }
                r_run += (double)rel;
            } else {
                // Some columns of the block are re-based: their score is the dense product q . k_hat(j) (Eq. 4
                // telescoped), taken from the K_hat Q^T tile; the running score continues from it.
                const f32x16 tile = rebase_tile(blk);
                const uint32_t mybits = half ? (dm >> 4) : dm;   // bit 8q + bb: this lane's column 4q + bb is re-based
                float w[16], t_own[4], t_oth[4];
                bool ab[16];                                     // w holds an absolute score (a re-base came before)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float run = 0.f;
                    bool absolute = false;
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        const bool rb = (mybits >> (8 * q + bb)) & 1u;
                        run = rb ? tile[4 * q + bb] : run + uu[4 * q + bb];
                        absolute = absolute || rb;
                        w[4 * q + bb] = run;
                        ab[4 * q + bb] = absolute;
                    }
                    t_own[q] = run;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) t_oth[q] = __shfl_xor(t_own[q], 32);
                float base = (float)r_run;                       // running score before the block's next group pair
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool f0 = (dm >> (8 * q)) & 0xfu, f1 = (dm >> (8 * q + 4)) & 0xfu;   // wave-uniform
                    const float g0 = half ? t_oth[q] : t_own[q], g1 = half ? t_own[q] : t_oth[q];
                    const float after0 = f0 ? g0 : base + g0;    // ... after lane half 0's group of four columns
                    const float after1 = f1 ? g1 : after0 + g1;  // ... after lane half 1's
                    const float mine = half ? after0 : base;
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) s[4 * q + bb] = ab[4 * q + bb] ? w[4 * q + bb] : mine + w[4 * q + bb];
                    base = after1;
                }
                r_run = (double)base;
            }
            softmax_pv(s, far_scale, vreg);
        };

        // Per block b: every wave gathers its four columns (G), the updates cross the work group through the exchange
        // buffer (two barriers), and every wave turns the updates of its 32 score rows into scores, softmax and P V (S).
        // S of block b is run during iteration b + 1, by the first wave of each SIMD before its gather and by the
        // second one after it, so that on every SIMD the matrix-core / exponential phase of one wave meets the LDS-bound
        // gather of the other instead of both waves idling through the same phases together.
        const bool late_s = wave >= kWaves / 2;                  // (waves w and w + 4 share a SIMD)
        float uu[16];
        uint32_t dm_prev = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) uu[r] = 0.f;
        for (int blk = f_lo; blk < f_hi; ++blk) {
            if (blk > f_lo && !late_s) {
                u32x4 vreg[2 * MT];
                load_v(vreg, (blk - 1) * kTB);
                scores_softmax_pv(blk - 1, uu, dm_prev, vreg);
            }
            w_store(st, pk_cur);                                 // this block's chunks into the ring
            const u32x3 pk = pk_cur;
            pk_cur = pk_nxt;
            g_issue(st, blk + 1, pk_cur);                        // next block's chunks into registers
            pk_nxt = pack_of(blk + 2);
            const uint32_t dm = pk[2];                           // re-based columns of this block (wave-uniform)
            if (dm) load_h_piece(blk);
            gather_block(pk);
            if (blk > f_lo && late_s) {
                u32x4 vreg[2 * MT];
                load_v(vreg, (blk - 1) * kTB);
                scores_softmax_pv(blk - 1, uu, dm_prev, vreg);
            }
            if (dm) park_h_piece(blk);                           // (its buffer was last read by S of block b - 2)
            lds_barrier();                                       // u of this block complete
            const float *up = ubuf + (4 * half) * kRows + my_sr;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) uu[4 * q + bb] = up[(8 * q + bb) * kRows];
            dm_prev = dm;
            lds_barrier();                                       // u buffer free for the next block
        }
        {
            u32x4 vreg[2 * MT];
            load_v(vreg, (f_hi - 1) * kTB);
            scores_softmax_pv(f_hi - 1, uu, dm_prev, vreg);
        }
    }

    // ---------------------------------------------------------------- near blocks (and all blocks in rebase mode)
    // Exact scores K Q^T (and K_hat Q^T where needed) on the matrix cores.  The K / K_hat / V tiles of a
    // block are fetched once per work group, one 16-byte piece per thread, a block ahead into registers,
    // then parked in LDS in operand order (lane-contiguous 16-byte slots, conflict free) where all 8 waves
    // read them.  Three LDS buffers rotate (tiles are requested two blocks ahead); one barrier per block.
    if (n_lo < n_hi) {
        u32x4 qreg[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[ks] = *(const u32x4 *)(my_q + ks * 16 + half * 8);
        constexpr int kTileBytes = D * 64;                       // 32 keys x D channels, bf16
        constexpr int kPieces = kTileBytes / 16;                 // 16-byte pieces per tile (256 or 512)
        char *tiles = lds_raw + kQtBytes;                        // [3 buffers][K, K_hat, V]
        // Every thread loads a piece - at head_dim 64, where a tile has only 256, the upper half of the work group
        // loads the lower half's pieces again and does not store them: loads that sit under a condition make the
        // compiler wait for every load in flight before a piece is parked, the younger set's included.
        const bool has_piece = kPieces == 512 || tid < kPieces;
        const int ptid = tid & (kPieces - 1);
        // K piece of thread ptid: key row ptid % 32, 8-channel segment ptid / 32.  Its operand-order slot is then
        // ptid itself, so a wave's 64 LDS stores are contiguous (a row-major thread-to-piece map made 16 lanes
        // hit the same banks)
        const int pr = ptid & 31, pseg = ptid >> 5;
        const int kslot = ((pseg >> 1) * 64 + (pseg & 1) * 32 + pr) * 16;
        // operand X of a block: K_hat while every row has the block outside its window (rebase mode), else K
        auto first_src = [&](int jb) -> const bf16_t * { return (jb + kTB <= win_first) ? Hp : Kp; };
        struct Pieces {
            u32x4 k, h, v;
        };
        auto load_tiles = [&](Pieces &pc, int blk) {
            const int jb = blk * kTB;
            const size_t roff = (size_t)min(jb + pr, n - 1) * D + pseg * 8;
            pc.k = *(const u32x4 *)(first_src(jb) + roff);
            if (!kAligned) pc.h = *(const u32x4 *)(Hp + roff);   // unconditional unless the tile cannot exist
            pc.v = *((const u32x4 *)Vtp + (size_t)blk * kPieces + ptid);
        };
        auto store_tiles = [&](const Pieces &pc, int buf) {
            char *base = tiles + buf * (3 * kTileBytes);
            if (has_piece) {
                *(u32x4 *)(base + kslot) = pc.k;
                if (!aligned) *(u32x4 *)(base + kTileBytes + kslot) = pc.h;
                *(u32x4 *)(base + 2 * kTileBytes + ptid * 16) = pc.v;
            }
        };
        // transposed score tile S^T[key][score row] = X[jb + key] . q, X tile in operand order at xt (a per-lane
        // address: tile base + 16 * lane, so that every read below is that address plus a constant)
        auto score_tile = [&](const char *xt) -> f32x16 {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const u32x4 xa = *(const u32x4 *)(xt + ks * 1024);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(xa), as_bf16x8(qreg[ks]), acc, 0, 0, 0);
            }
            return acc;
        };
        // raw score registers of a block: exact / K_hat scores picked per element, causal mask applied
        auto block_scores = [&](float (&s)[16], const char *base, int jb) {
            {
                const f32x16 sk = score_tile(base);
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = sk[r];
            }
            if (!aligned && first_src(jb) == Kp && jb < win_last) {
                // some row has part of the block left of its window: exact score inside the row's own
                // window, K_hat score (telescoped Eq. 4) left of it
                const f32x16 sh = score_tile(base + kTileBytes);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = jb + 8 * (r >> 2) + 4 * half + (r & 3);
                    s[r] = (j >= my_win) ? s[r] : sh[r];
                }
            }
            if (jb + kTB > i0 + 1) {   // some entry is masked for some row of the tile
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = jb + 8 * (r >> 2) + 4 * half + (r & 3);
                    s[r] = (j <= my_i) ? s[r] : -INFINITY;
                }
            }
        };
        // Software pipeline over blocks: the score MFMAs of block b+1 are issued before the softmax of
        // block b, so matrix-core and vector-ALU work of one wave overlap.  Buffer b % 3 holds the tiles of
        // block b; its K tile is read one iteration before its V tile.
        // Two register sets of pieces alternate: a set is parked in LDS and at once re-used for the block two
        // further on, so no set is ever copied (a copy of registers that a load is still filling waits for it).
        // Loads and stores are issued every iteration, past the last block too (clamped to it: a dead buffer gets
        // a copy nobody reads), so that the number of loads in flight is the same on every path and the wait
        // before a set is parked lets the younger set's loads stay in flight.
        Pieces pa, pb;
        load_tiles(pa, n_lo);
        load_tiles(pb, min(n_lo + 1, n_hi - 1));
        lds_barrier();                                           // the far loop's LDS use is over
        store_tiles(pa, 0);
        load_tiles(pa, min(n_lo + 2, n_hi - 1));
        lds_barrier();
        float s_a[16], s_b[16];                                  // raw scores of the current / the next block, in turn
        const char *lane_tiles = tiles + lane * 16;              // per-lane view of the tile buffers
        block_scores(s_a, lane_tiles, n_lo * kTB);
        int buf = 0;
        // one block: `next` holds the pieces of block blk + 1, s_cur this block's scores, s_next receives the next one's
        auto do_block = [&](int blk, Pieces &next, float (&s_cur)[16], float (&s_next)[16]) {
            const char *base = lane_tiles + buf * (3 * kTileBytes);
            const int nbuf = buf == 2 ? 0 : buf + 1;
            store_tiles(next, nbuf);
            load_tiles(next, min(blk + 3, n_hi - 1));            // in flight for two iterations
            lds_barrier();                                       // LDS only: the tile loads stay in flight
            if (blk + 1 < n_hi) block_scores(s_next, lane_tiles + nbuf * (3 * kTileBytes), (blk + 1) * kTB);
            u32x4 vreg[2 * MT];
#pragma unroll
            for (int k = 0; k < 2 * MT; ++k) vreg[k] = *(const u32x4 *)(base + 2 * kTileBytes + k * 1024);
            softmax_pv(s_cur, a.scale_log2, vreg);
            buf = nbuf;
        };
        // everything requested so far has landed before the loop is entered: the wait at its head then only has to
        // cover what the previous trip left in flight (the compiler sizes it for the worse of both ways in)
        __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)
        for (int blk = n_lo; blk < n_hi; blk += 2) {
            do_block(blk, pb, s_a, s_b);
            if (blk + 1 < n_hi) do_block(blk + 1, pa, s_b, s_a);
        }
    }

    // ---------------------------------------------------------------- epilogue
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (geo.parts > 1) {
        // one part of a split tile: unnormalised output rows, running maximum and sum for prefill_merge_kernel
        // (rows past the end of the sequence are written too, as they stand, and never read: the stores stay whole)
        // Pieces of 4 channels in the order the accumulators hold them - piece (wave, mt, q4, lane) = score row
        // 32 wave + lane % 32, channels 32 mt + 8 q4 + 4 (lane / 32) .. + 3 - so that every store instruction of a
        // wave writes 1 KiB in one run.
        const size_t slot = ((size_t)(unit * a.hgroups + hchunk) * a.tiles + tile) * a.ksplit + seg;
        f32x4 *po = (f32x4 *)(a.part_o + slot * kRows * D) + (size_t)wave * (MT * 4 * 64) + lane;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                po[(mt * 4 + q4) * 64] = f32x4{oacc[mt][4 * q4 + 0], oacc[mt][4 * q4 + 1], oacc[mt][4 * q4 + 2],
                                               oacc[mt][4 * q4 + 3]};
        if (half == 0) *(f32x2 *)(a.part_ml + (slot * kRows + my_sr) * 2) = f32x2{m_run, l_tot};
        return;
    }
    if (my_valid) {
        const float inv = 1.f / l_tot;
        bf16_t *orow = a.O + (((size_t)b * a.Hq + head0 + my_hh) * a.nq + (my_i - a.q_off)) * D;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w;
                w[0] = pack_bf16x2(oacc[mt][4 * q4 + 0] * inv, oacc[mt][4 * q4 + 1] * inv);
                w[1] = pack_bf16x2(oacc[mt][4 * q4 + 2] * inv, oacc[mt][4 * q4 + 3] * inv);
                *(u32x2 *)(orow + mt * 32 + 8 * q4 + 4 * half) = w;
            }
    }
}

// Second launch of a split attention launch: the parts of every tile that was cut (TileGeometry::parts > 1) are
// merged flash-decoding style - with M the largest running maximum, O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s -
// and the output rows written.  One work group per (tile, wave slab of 32 score rows); a thread on pieces of 4
// channels, all parts of a piece loaded at once (indices clamped, the surplus weighted 0: no load sits under a
// condition, so they are all in flight together).
constexpr int kMaxSplit = 8;
template <int D, bool kGather>
__global__ __launch_bounds__(256) void prefill_merge_kernel(MfmaArgs a) {
    constexpr int MT = D / 32, kSlab = MT * 4 * 64;          // pieces of one wave's 32 score rows
    const int t = blockIdx.x / kWaves, wv = blockIdx.x % kWaves;   // t = (unit * hgroups + hchunk) * tiles + tile
    const int tile = t % a.tiles, uh = t / a.tiles, hchunk = uh % a.hgroups, unit = uh / a.hgroups;
    const TileGeometry geo = tile_geometry<kGather>(a, tile);
    if (geo.parts <= 1) return;                              // that tile's one work group has written its rows itself
    const int b = unit / a.Hkv, hk = unit % a.Hkv, g = a.Hq / a.Hkv, head0 = hk * g + hchunk * a.GH;
    const float *po = a.part_o + (size_t)t * a.ksplit * kRows * D;
    const float *pml = a.part_ml + (size_t)t * a.ksplit * kRows * 2;
    for (int k = threadIdx.x; k < kSlab; k += 256) {
        // piece of a part's output, in the order the attention kernel stored it (see its epilogue)
        const int idx = wv * kSlab + k, ln = k & 63, slot = k >> 6;
        const int sr = 32 * wv + (ln & 31), ch = 32 * (slot >> 2) + 8 * (slot & 3) + 4 * (ln >> 5);
        const int hh = sr / a.RT, i = geo.i0 + sr - hh * a.RT;
        f32x2 ml[kMaxSplit];
        f32x4 o[kMaxSplit];
#pragma unroll
        for (int p = 0; p < kMaxSplit; ++p) {
            const size_t pe = (size_t)min(p, geo.parts - 1);
            ml[p] = *(const f32x2 *)(pml + (pe * kRows + sr) * 2);
            o[p] = *(const f32x4 *)(po + pe * kRows * D + (size_t)idx * 4);
        }
        if (i >= a.n) continue;
        float M = -INFINITY;
#pragma unroll
        for (int p = 0; p < kMaxSplit; ++p)
            if (p < geo.parts) M = fmaxf(M, ml[p][0]);
        float L = 0.f;
        f32x4 O = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < kMaxSplit; ++p) {
            // (part 0 holds key 0, which every row sees: M is finite; a part none of whose keys a row sees has m = -inf)
            const float w = (p >= geo.parts || ml[p][0] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[p][0] - M);
            L = w == 0.f ? L : fmaf(w, ml[p][1], L);
#pragma unroll
            for (int e = 0; e < 4; ++e) O[e] = w == 0.f ? O[e] : fmaf(w, o[p][e], O[e]);   // (unread rows may hold anything)
        }
        const float inv = 1.f / L;
        u32x2 w2;
        w2[0] = pack_bf16x2(O[0] * inv, O[1] * inv);
        w2[1] = pack_bf16x2(O[2] * inv, O[3] * inv);
        *(u32x2 *)(a.O + (((size_t)b * a.Hq + head0 + hh) * a.nq + (i - a.q_off)) * D + ch) = w2;
    }
}

// tiles of a launch: row tiles x head chunks x units; GH heads of RT rows make a tile's kRows score rows
static void tile_counts(const PrefillArgs &p, int &GH, int &RT, int &tiles, int &hgroups) {
    const int g = p.Hq / p.Hkv;
    GH = (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
    RT = kRows / GH;
    tiles = (p.nq + RT - 1) / RT;
    hgroups = g / GH;
}

template <int D>
static void launch_d(const PrefillArgs &p, void *vt, int n_pad, hipStream_t s) {
    const int units = p.B * p.Hkv;
    const int ld = p.ld > 0 ? p.ld : p.n, ld_pad = p.ld > 0 ? prefill_mfma_n_pad(p.ld) : n_pad;
    if (!p.fused && p.vt_from < n_pad / kTB)
        hipLaunchKernelGGL((transpose_v_kernel<D>), dim3(n_pad / kTB - p.vt_from, units), dim3(256), 0, s,
                           (const bf16_t *)p.V, (bf16_t *)vt, p.n, ld, ld_pad, p.vt_from);
    MfmaArgs a;
    a.ld = ld;
    a.ld_pad = ld_pad;
    a.V = (const bf16_t *)p.V;
    a.mask_bits = p.mask_bits;
    a.nnz = (unsigned long long *)p.nnz;
    a.counts = const_cast<uint32_t *>(p.counts);
    a.nch8 = const_cast<uint8_t *>(p.nch8);
    a.theta = p.theta;
    a.Q = (const bf16_t *)p.Q;
    a.K = (const bf16_t *)p.K;
    a.Khat = (const bf16_t *)p.Khat;
    a.Vt = (const bf16_t *)vt;
    a.O = (bf16_t *)p.O;
    a.ents = (const EntryChunk *)p.ents;
    a.plan = (const uint8_t *)p.plan;
    a.dense = p.dense;
    a.Hq = p.Hq;
    a.Hkv = p.Hkv;
    a.n = p.n;
    a.n_pad = n_pad;
    a.W = p.W;
    a.rebase = p.rebase;
    a.sliding = p.sliding;
    tile_counts(p, a.GH, a.RT, a.tiles, a.hgroups);
    a.q_off = p.q_off;
    a.nq = p.nq;
    a.scale_log2 = p.scale_log2;
    a.ksplit = (!p.fused && !p.rebase && p.ksplit > 1 && p.part) ? p.ksplit : 1;
    a.parts_total = 0;
    for (int t = 0; t < a.tiles; ++t)
        a.parts_total += tile_geometry_of(a.q_off, a.RT, a.n, a.W, a.sliding, a.ksplit, !p.rebase, t).parts;

    a.part_o = (float *)p.part;
    a.part_ml = a.part_o + (size_t)units * a.tiles * a.hgroups * a.ksplit * kRows * D;
    const size_t lds_far = (size_t)kTB * kRows * 4 + (size_t)kWaves * (4 * (D / kGroup) * 64 + 4 * 64) +
                           (size_t)2 * D * 64;                  // u exchange, entry rings, two fp16 K_hat tiles
    const size_t lds_near = (size_t)9 * D * 64;
    const size_t lds_gather = (size_t)D * kRows * 2 + (lds_far > lds_near ? lds_far : lds_near);
    // fused_prepare's scratch: LDS copies of up to kFusedMaxElems key elements, or the per-wave V tiles
    const size_t lds_prep = fused_lds_bytes(D, kFusedMaxElems / D) > (size_t)64 + kWaves * kTB * (D + 2) * 2
                                ? fused_lds_bytes(D, kFusedMaxElems / D) : (size_t)64 + kWaves * kTB * (D + 2) * 2;
    const size_t lds_fused_gather = lds_gather > lds_prep ? lds_gather : lds_prep;
    const size_t lds_fused_rebase = lds_near > lds_prep ? lds_near : lds_prep;
    static std::atomic<uint64_t> lds_set[6];                     // per instantiation of launch_d, one bit per device
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, true, false, true>, (int)lds_fused_gather, lds_set[4]);
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, false, false, true>, (int)lds_fused_rebase, lds_set[5]);
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, true, false>, (int)lds_gather, lds_set[0]);
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, true, true>, (int)lds_gather, lds_set[1]);
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, false, false>, (int)lds_near, lds_set[2]);
    ensure_dynamic_lds((const void *)prefill_mfma_kernel<D, false, true>, (int)lds_near, lds_set[3]);
    const size_t blocks = (size_t)units * a.parts_total * a.hgroups;
    // XCD-aware order needs units * xsplit parts to deal out evenly over 8 XCDs and a unit to split evenly
    a.xsplit = 0;
    for (int sp = 1; sp <= 8; sp *= 2)
        if ((units * sp) % 8 == 0) {
            if ((a.parts_total * a.hgroups) % sp == 0 && sp < 8) a.xsplit = sp;
            break;
        }
    // every tile's rows (RT consecutive positions from q_off on) lie in one window square whose start is a multiple
    // of the block size
    const bool all_aligned = !p.sliding && p.W % kTB == 0 && p.W % a.RT == 0 && p.q_off % a.RT == 0;
    const dim3 grid((unsigned)blocks), block(512);
    if (p.fused && p.rebase)
        hipLaunchKernelGGL((prefill_mfma_kernel<D, false, false, true>), grid, block, lds_fused_rebase, s, a);
    else if (p.fused)
        hipLaunchKernelGGL((prefill_mfma_kernel<D, true, false, true>), grid, block, lds_fused_gather, s, a);
    else if (p.rebase && all_aligned)
        hipLaunchKernelGGL((prefill_mfma_kernel<D, false, true>), grid, block, lds_near, s, a);
    else if (p.rebase)
        hipLaunchKernelGGL((prefill_mfma_kernel<D, false, false>), grid, block, lds_near, s, a);
    else if (all_aligned)
        hipLaunchKernelGGL((prefill_mfma_kernel<D, true, true>), grid, block, lds_gather, s, a);
    else
        hipLaunchKernelGGL((prefill_mfma_kernel<D, true, false>), grid, block, lds_gather, s, a);
    if (a.ksplit > 1) {
        const dim3 mgrid((unsigned)(units * a.tiles * a.hgroups * kWaves));
        if (p.rebase)
            hipLaunchKernelGGL((prefill_merge_kernel<D, false>), mgrid, dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL((prefill_merge_kernel<D, true>), mgrid, dim3(256), 0, s, a);
    }
}

// A launch with fewer than four tiles per compute unit is cut along the keys, as many ways (a power of two, at most
// 8) as bring it there, one with fewer than eight in two; never more parts than the longest tile has runs of
// kSplitMinBlocks key blocks.
int prefill_mfma_ksplit(const PrefillArgs &p) {
    if (p.fused || p.rebase || !prefill_mfma_supported(p)) return 1;   // (matrix-core blocks are too cheap to pay for it)
    int GH, RT, tiles, hgroups;
    tile_counts(p, GH, RT, tiles, hgroups);
    const long long groups = (long long)p.B * p.Hkv * tiles * hgroups, want = 4LL * device_cu_count();
    int ks = 1;
    while (ks < kMaxSplit && groups * ks < want) ks *= 2;
    // (measured: going from whole tiles to halves still pays at 5 tiles per CU - 4 x 20 heads x 4096 tokens: 2.60 ->
    // 2.32 ms, the long tiles' tail - but not at 10, 8192 tokens: 8.05 -> 8.72 ms; and cuts finer than `want` asks for
    // cost more than they balance)
    if (ks == 1 && groups < 2 * want) ks = 2;
    const int longest = (p.q_off + p.nq - 1) / kTB + 1;      // key blocks of the last tile
    while (ks > 1 && longest / kSplitMinBlocks < ks) ks /= 2;
    return ks;
}

size_t prefill_mfma_part_bytes(const PrefillArgs &p, int ksplit) {
    if (ksplit <= 1) return 0;
    int GH, RT, tiles, hgroups;
    tile_counts(p, GH, RT, tiles, hgroups);
    return (size_t)p.B * p.Hkv * tiles * hgroups * ksplit * kRows * (p.d + 2) * sizeof(float);
}

int prefill_mfma_n_pad(int n) { return (n + 63) / 64 * 64; }

bool prefill_mfma_supported(const PrefillArgs &p) {
    return p.dtype == 1 && (p.d == 64 || p.d == 128) &&
           (size_t)p.B * p.Hkv * ((p.n + 63) / 64) * (p.Hq / p.Hkv) < ((size_t)1 << 31);
}

void launch_prefill_mfma(const PrefillArgs &p, void *vt, hipStream_t s) {
    const int n_pad = prefill_mfma_n_pad(p.n);
    if (p.d == 64)
        launch_d<64>(p, vt, n_pad, s);
    else
        launch_d<128>(p, vt, n_pad, s);
}

}  // namespace da
