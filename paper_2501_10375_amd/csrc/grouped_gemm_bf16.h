// Grouped bf16 GEMM for the expert FFN on the CDNA4 matrix cores (device code).
//
// Computes, per (expert, slot tile of BT = 256 or 128 slots, feature tile),
//   NMAT = 2 (gemm1): act[slot, f] = silu(tok[slot] . wa[e, f]) * (tok[slot] . wb[e, f])   (bf16 out)
//   NMAT = 1 (gemm2): out[slot, n] = tok[slot] . wa[e, n]                                  (fp32 out)
// where tok rows are gathered rows of x (gemm1) or rows of act (gemm2), and every
// operand is K-contiguous ("row . row" contraction, no transposes anywhere).
//
// Organisation (gfx950):
//   * Tile BT slots x 256 weight rows (NMAT = 2: 128 features of each matrix), K in steps of BK.
//     WT x WW wavefronts (slot groups x weight-row groups); each owns (BT/WT) x (256/WW) outputs
//     as v_mfma_f32_32x32x16_bf16 tiles.  Weights are the MFMA "A" operand, slot rows the "B"
//     operand, so a lane ends up holding 4 consecutive output features of one slot.
//   * Operand tiles go HBM/L2 -> LDS directly (global_load_lds_dwordx4, no register staging), in a
//     ring of STAGES tiles.  Each lane supplies its own global address, which is how gathered rows
//     and the XOR swizzle are expressed: the 16-byte piece that must land at LDS position p is
//     fetched by the lane whose data lands at p.  The swizzle makes the ds_read_b128 operand reads
//     bank-conflict free on the 64-bank LDS.
//   * The loads are issued from inline asm so the compiler does not serialise them against the
//     LDS reads of other stages; completion is enforced by hand: s_waitcnt vmcnt(n) on the issuing
//     wavefront, then a workgroup barrier, before any wavefront reads the stage.  One barrier per
//     K step.  Inside a step MFMAs, LDS reads and loads are interleaved one for one.
//   * Persistent schedule, one workgroup per CU, tiles handed out in rounds per XCD so the
//     workgroups of an XCD share operand tiles through its L2; the last, partial round is split
//     along K so that all CUs stay busy (see persistent()).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "bf16_utils.h"

namespace moe {
namespace gg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kBT = 256;   // most slots per tile (the template parameter BT is 256 or 128)
constexpr int kBW = 256;   // weight rows per tile (all matrices together)
constexpr int kXcds = 8;
constexpr int kMaxWgsPerXcd = 32;  // persistent grid: at most 8 x 32 workgroups
constexpr int kMaxSplit = 4;       // K parts of a tile in the last round (the sum of the pieces costs as much as 1/16 tile each)

// Layout of the int32 `sync` block a GEMM launch uses (all zero when the kernel starts):
//   [0, 8)                      tiles handed out so far in each XCD (see persistent())
//   [8, 8 + 8 * 32)             arrival counter of each split tile (XCD-major)
constexpr int kSyncInts = kXcds + kXcds * kMaxWgsPerXcd;
// fp32 scratch for split tiles: one 256 x 256 partial accumulator tile per workgroup.
constexpr int kMaxBT = 256;  // tallest slot tile any flavour uses
constexpr size_t kPartialFloats = (size_t)kMaxBT * kBW;
constexpr size_t kScratchBytes = (size_t)kXcds * kMaxWgsPerXcd * kPartialFloats * sizeof(float);

// Tile list.  The number of real tiles depends on the routing (sum over experts of
// ceil(count / 256) slot tiles, times the feature tiles) and is only known on the device, so
// every workgroup derives it from `offs`.  Tile order: expert, group of kGroup slot tiles, feature
// tile, slot tile within the group.  32 consecutive tiles (what the 32 CUs of one XCD work on at
// one time) are then about 8 slot tiles x 4 feature tiles of one expert: 12 distinct operand tiles
// feed 32 workgroups through the XCD's L2.
constexpr int kGroup = 8;

__device__ inline int count_tiles(const int32_t* __restrict__ offs, int E, int n_ftiles, int bt, int& slot_tiles) {
    int total = 0;
    for (int i = 0; i < E; ++i) total += (offs[i + 1] - offs[i] + bt - 1) / bt;
    slot_tiles = total;
    return total * n_ftiles;
}

__device__ inline void tile_of(const int32_t* __restrict__ offs, int E, int n_ftiles, int bt, int id, int& e, int& slot0,
                               int& rows, int& ft) {
    int acc = 0;
    e = 0; slot0 = 0; rows = 1; ft = 0;
    for (int i = 0; i < E; ++i) {
        const int c = offs[i + 1] - offs[i];
        const int mt = (c + bt - 1) / bt;
        const int tiles = mt * n_ftiles;
        if (id < acc + tiles) {
            const int local = id - acc;
            const int grp = local / (kGroup * n_ftiles);  // full groups come first
            const int in_grp = local - grp * (kGroup * n_ftiles);
            const int gsize = min(kGroup, mt - grp * kGroup);
            ft = in_grp / gsize;
            const int m = grp * kGroup + (in_grp - ft * gsize);
            e = i;
            slot0 = offs[i] + m * bt;
            rows = min(bt, c - m * bt);
            return;
        }
        acc += tiles;
    }
}

// 16 bytes per lane from `gptr` to LDS byte address lds_base + lane * 16 (lds_base wave-uniform).
// (The compiler does not insert hazard wait states inside inline asm: an LDS-DMA load that reads M0
// needs one after the scalar write of M0, hence the s_nop.)
__device__ inline void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// 16-byte store that is written through to memory (device scope), as an agent-scope atomic store is.
// The compiler does not track hazards of instructions inside inline asm: a store of more than 8
// bytes needs a wait state before its data registers may be overwritten, hence the s_nop.
__device__ inline void store16_through(float* p, f32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}

// Workgroup barrier that orders LDS traffic only (no wait on outstanding global loads).
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// LDS swizzle: the 16-byte piece `chunk` of tile row `row` is stored at piece position
// piece(row, chunk) of that row.  The LDS has 64 four-byte banks (256 bytes per cycle), so a
// ds_read_b128 serves 16 lanes per cycle; the lanes of one MFMA operand read sit on 16
// consecutive rows at the same chunk, and the XOR below spreads them over all 64 banks.
template <int BK>
struct Swz;
template <>
struct Swz<64> {  // 128-byte rows, 8 pieces; two rows span the 64 banks
    static __device__ inline int piece(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }
};
template <>
struct Swz<32> {  // 64-byte rows, 4 pieces; four rows span the 64 banks
    static __device__ inline int piece(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }
};

// SKIP: slot fragments of a ragged tile that hold no valid slot are skipped (their LDS reads and
// MFMAs).  That pays when many experts are cold (most tiles ragged), but it puts every MFMA behind a
// scalar branch, which costs a little when nearly all tiles are full; the launcher decides.
// ALT (gemm1 only): a slot's row comes from `tok_alt` instead of `tok_base` when alt_mask[assignment]
// is set: expert execution with some selections pre-calculated on an earlier hidden state.
//
// W3: three weight stages and two slot stages (160 KB of LDS) instead of STAGES stages of both.  With two
// stages of both operands a K step's loads can only be requested after the barrier that starts the K
// step before, all at once: the 64 load instructions of a workgroup then queue in the CU's address
// path for about a thousand cycles, and the MFMAs interleaved with them are held back as long (a
// wavefront issues in order).  Weight lines are the ones that come from memory, slot lines mostly
// from the L2 or the memory-side cache; so the weights get the third stage: they are requested two K
// steps ahead and their load instructions are spread evenly over a K step, and only the slot loads
// (half the instructions) remain tied to the barrier.  Stage offsets rotate at run time (scalar
// registers), so the loop body is one K step and needs few address registers.
template <int NMAT, int BK, int STAGES, int WT, int WW, bool SKIP, int BT = kBT, bool ALT = false, bool W3 = false>
struct Gemm {
    static_assert(!W3 || (STAGES == 2 && BK == 64 && BT == kBT && !SKIP), "the three-weight-stage flavour is built for full tiles");
    static_assert(!ALT || NMAT == 2, "only the first GEMM gathers rows of x");
    static constexpr int kWaves = WT * WW;                     // WT slot groups x WW weight-row groups
    static constexpr int kThreads = kWaves * 64;
    static_assert(BT % (32 * WT) == 0 && BT <= kMaxBT, "slot tile height");
    static constexpr int kTF = BT / WT / 32;                   // 32-slot MFMA tiles per wavefront
    static constexpr int kWF = 256 / WW / 32;                  // 32-row weight MFMA tiles per wavefront
    static constexpr int kTokStageRows = BT / kWaves;          // slot rows a wavefront stages
    static constexpr int kStageRows = 256 / kWaves;            // weight rows a wavefront stages
    static_assert(kWF % NMAT == 0, "a wavefront needs the same features of every matrix");
    static constexpr int kRowBytes = BK * 2;
    static constexpr int kTokTileBytes = BT * kRowBytes;       // the slot tile of one stage
    static constexpr int kTileBytes = 256 * kRowBytes;         // the weight tile of one stage
    static constexpr int kStageBytes = kTokTileBytes + kTileBytes;  // slots, then weights
    static constexpr int kLdsBytes = W3 ? 3 * kTileBytes + 2 * kTokTileBytes : STAGES * kStageBytes;
    static constexpr int kRowsPerLoad = 1024 / kRowBytes;      // rows covered by one wavefront-wide 1 KB load
    static_assert(kTokStageRows % kRowsPerLoad == 0, "whole loads per wavefront");
    static constexpr int kLoadsTok = kTokStageRows / kRowsPerLoad;  // slot loads per thread per stage
    static constexpr int kLoadsPerOperand = kStageRows / kRowsPerLoad;  // weight loads per thread per stage
    static constexpr int kLoads = kLoadsTok + kLoadsPerOperand;
    static constexpr int kPieces = kRowBytes / 16;
    static constexpr int kKSteps = BK / 16;
    static constexpr int kBF = kBW / NMAT;                     // features per tile (per matrix)
    static constexpr int kFragsPerMat = kWF / NMAT;
    static constexpr int kFeatPerWave = 32 * kFragsPerMat;
    static_assert(kLdsBytes >= 65536, "the epilogue transposes 64 KB through LDS");
    // Start of the stage that a tile's prologue leaves alone (its first load arrives after the first barrier).
    static constexpr int kHandoffOffset = W3 ? 3 * kTileBytes + kTokTileBytes : (STAGES - 1) * kStageBytes;

    // tok_base: gemm1 -> x [T, K] rows gathered via row_of_slot / topk; gemm2 -> act [A, K] rows = slots.
    // wa, wb: [E, N, K]; dst: gemm1 -> bf16 [A, N]; gemm2 -> fp32 [A, N].
    //
    // Persistent schedule: the grid is one workgroup per CU.  Workgroup b belongs to XCD b % 8 (the
    // hardware deals workgroups round-robin to the XCDs) and is its member b / 8.  An XCD works
    // through the tile list in rounds of `members` consecutive tiles, so that its workgroups work on
    // tiles that share operand lines at about the same time and most lines are pulled into the
    // XCD's L2 once per round instead of once per workgroup.  A workgroup starts with the tile of
    // its member number and then takes the XCD's next tile from a counter whenever it has finished
    // one: tiles differ in cost (ragged slot tiles skip the MFMAs of their empty fragments, tiles
    // of cold experts wait for memory), and nobody waits for anybody.  Letting the members drift
    // apart by a fraction of a K step is also faster than holding them in step, because fewer of
    // them then ask for the same line at the same moment.
    //
    // The last round usually has fewer tiles than members (`rem`).  Each of its tiles is then split
    // along K into `parts` = min(kMaxSplit, members / rem) pieces handed out like tiles.
    // Every piece is written to `scratch` as a raw accumulator tile; the workgroup that arrives last
    // at the tile's counter adds the pieces in part order (so the result does not depend on who that
    // is) and runs the normal epilogue.
    static __device__ void persistent(const uint16_t* __restrict__ tok_base, const uint16_t* __restrict__ wa,
                                      const uint16_t* __restrict__ wb, const int32_t* __restrict__ offs,
                                      const int32_t* __restrict__ row_of_slot, int E, int topk, int N, int K,
                                      void* __restrict__ dst, int32_t* __restrict__ sync,
                                      float* __restrict__ scratch, unsigned char* lds,
                                      const uint16_t* __restrict__ tok_alt = nullptr,
                                      const uint8_t* __restrict__ alt_mask = nullptr) {
        const int n_ftiles = (N + kBF - 1) / kBF;
        int slot_tiles;
        const int total = count_tiles(offs, E, n_ftiles, BT, slot_tiles);
        // Ragged tiles issue only the MFMAs of their valid fragments when more than an eighth of the slot
        // tiles' rows is padding.  A tile that finishes early sends its workgroup ahead of the others of
        // its round, which then share fewer operand lines in the L2: with little padding (4096 tokens of
        // the Mixtral shape: 9 %) that buys under 1 % of time for two thirds more memory traffic, with
        // much (2048 tokens: 25 %) it is 5-6 % faster.
        const int routed = offs[E] - offs[0];
        const bool short_loops = (slot_tiles * BT - routed) * 8 > slot_tiles * BT;
        const int KT = K / BK;
        const int xcd = blockIdx.x % kXcds, member = blockIdx.x / kXcds;
        const int members = min((int)gridDim.x / kXcds, kMaxWgsPerXcd);
        if (member >= members) return;
        // Full rounds: round r of XCD x is tiles [(r * 8 + x) * members, +members) of the list, so the
        // XCDs take turns along the list and each sees the same mix of heavy tiles (hot experts, full
        // slot tiles) and light ones (cold experts, whose rounds are bound by streaming their weights).
        // The tiles left over after the last full round of all XCDs are split evenly between the XCDs.
        const int per_super_round = kXcds * members;
        const int full_rounds = total / per_super_round;
        const int left = total - full_rounds * per_super_round;
        const int chunk = (left + kXcds - 1) / kXcds;
        const int rem = max(0, min(left, (xcd + 1) * chunk) - xcd * chunk);
        const int rem_first = full_rounds * per_super_round + xcd * chunk;
        const int parts = rem > 0 ? max(1, min(min(kMaxSplit, members / rem), KT / STAGES)) : 1;
        // Work items of this XCD in hand-out order: its whole tiles, then the pieces of its split tiles.
        const int n_whole = full_rounds * members;
        const int n_items = n_whole + rem * parts;
        int item = member;  // the counter hands out items `members`, `members` + 1, ...
        while (item < n_items) {
            const bool split = item >= n_whole;
            const int p = split ? parts : 1;
            const int q = item - n_whole;  // piece number (split tiles only)
            const int t = split ? q / p : item % members, part = split ? q - t * p : 0;
            const int tile_index = split ? rem_first + t : ((item / members) * kXcds + xcd) * members + t;
            int e, slot0, rows, ft;
            tile_of(offs, E, n_ftiles, BT, tile_index, e, slot0, rows, ft);
            const int kt0 = (int)((long)KT * part / p), kt1 = (int)((long)KT * (part + 1) / p);
            item = members + tile(tok_base, wa, wb, row_of_slot, topk, N, K, dst, lds, e, slot0, rows, ft, kt0, kt1, p, part,
                                  scratch + ((size_t)xcd * kMaxWgsPerXcd + (size_t)t * p) * kPartialFloats,
                                  sync + kXcds + xcd * kMaxWgsPerXcd + t, sync + xcd, tok_alt, alt_mask, short_loops);
        }
    }

    // One tile over K steps [kt_begin, kt_end).  parts == 1: a whole tile.  parts > 1: piece `part`
    // of a split tile; `partials` is where this tile's pieces live (piece p at p * kPartialFloats),
    // `arrivals` its zero-initialised counter.  Returns what `handed_out` (the XCD's count of items
    // taken beyond every member's first) held when this workgroup asked for its next item.
    static __device__ int tile(const uint16_t* __restrict__ tok_base, const uint16_t* __restrict__ wa,
                                const uint16_t* __restrict__ wb, const int32_t* __restrict__ row_of_slot, int topk,
                                int N, int K, void* __restrict__ dst, unsigned char* lds, int e, int slot0, int rows,
                                int ft, int kt_begin, int kt_end, int parts, int part, float* __restrict__ partials,
                                int32_t* __restrict__ arrivals, int32_t* __restrict__ handed_out,
                                const uint16_t* __restrict__ tok_alt, const uint8_t* __restrict__ alt_mask,
                                bool short_loops) {
        const int n0 = ft * kBF;
        const int tid = threadIdx.x, lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
        const int wt = wave % WT, wq = wave / WT;  // slot group, weight-row group
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

        // ---- staging addresses: this wavefront stages rows [wave, wave + 1) * kTokStageRows of the slot tile
        // and rows [wave, wave + 1) * kStageRows of the weight tile
        const int lrow = lane / kPieces;                       // row within a 1 KB load
        const int lpiece = lane % kPieces;                     // LDS piece position within the row
        const size_t k_first = (size_t)kt_begin * kRowBytes;   // byte offset of this piece's first K step
        const char* gp[kLoads];  // slot loads first, then weight loads
#pragma unroll
        for (int q = 0; q < kLoadsTok; ++q) {
            const int r = wave * kTokStageRows + q * kRowsPerLoad + lrow;  // row in the slot tile
            const int chunk = Swz<BK>::piece(r, lpiece);        // global piece that belongs at this position
            const int slot = slot0 + min(r, rows - 1);          // rows past the end re-read the last valid row
            const int assignment = (NMAT == 2) ? row_of_slot[slot] : 0;   // t * topk + j
            const int src = (NMAT == 2) ? assignment / topk : slot;
            const uint16_t* rows_from = (ALT && alt_mask[assignment] != 0) ? tok_alt : tok_base;
            gp[q] = reinterpret_cast<const char*>(rows_from + (size_t)src * K) + chunk * 16 + k_first;
        }
#pragma unroll
        for (int q = 0; q < kLoadsPerOperand; ++q) {
            const int r = wave * kStageRows + q * kRowsPerLoad + lrow;  // row in the 256-row weight tile
            const int chunk = Swz<BK>::piece(r, lpiece);
            // weight rows: NMAT == 2 -> rows 0..127 are wa features, 128..255 wb features
            const int mat = (NMAT == 2) ? (r >> 7) : 0;
            const int f = min(n0 + ((NMAT == 2) ? (r & 127) : r), N - 1);
            const uint16_t* wsrc = (mat == 0) ? wa : wb;
            gp[kLoadsTok + q] = reinterpret_cast<const char*>(wsrc + ((size_t)e * N + f) * K) + chunk * 16 + k_first;
        }
        const int KT = kt_end - kt_begin;  // K steps of this piece, numbered from 0 below
        const uint32_t stage_off_tok = (uint32_t)(wave * kTokStageRows * kRowBytes);
        const uint32_t stage_off_w = (uint32_t)(kTokTileBytes + wave * kStageRows * kRowBytes);

        f32x16 acc[kWF][kTF];  // [weight frag][slot frag]
#pragma unroll
        for (int j = 0; j < kWF; ++j)
#pragma unroll
            for (int i = 0; i < kTF; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

        // ---- operand read offsets (rows within an operand tile)
        const int frow = lane & 31, fhalf = lane >> 5;
        // Weight frag j: NMAT == 2 -> matrix j / kFragsPerMat, feature tile j % kFragsPerMat of this
        // wavefront's features [wq * kFeatPerWave, +kFeatPerWave); NMAT == 1 -> weight rows
        // wq * kFeatPerWave + 32 j.
        int trow[kTF], wrow[kWF];
#pragma unroll
        for (int i = 0; i < kTF; ++i) trow[i] = (i * WT + wt) * 32 + frow;
        // Slot fragments (32 slots each) are dealt to the slot groups round-robin, so the valid slots of
        // a ragged tile spread evenly over the wavefronts (and the SIMDs they sit on); fragments that lie
        // entirely past the tile's last slot are skipped: n_tf = this wavefront's fragments with valid slots.
        const int n_tf = __builtin_amdgcn_readfirstlane(min(kTF, max(0, (rows - wt * 32 + 32 * WT - 1) / (32 * WT))));
#pragma unroll
        for (int j = 0; j < kWF; ++j)
            wrow[j] = (j / kFragsPerMat) * 128 * (NMAT - 1) + wq * kFeatPerWave + (j % kFragsPerMat) * 32 + frow;

        if constexpr (W3) {
            // A fragment read of row r, k16 step ks from a stage at byte offset `off` is at
            //   r * 128 + ((ks * 2 + fhalf) ^ ((r >> 1) & 7)) * 16 + off  =  base(r) ^ (ks << 5) ^ off,
            // base(r) = r * 128 + ((((r >> 1) & 7) ^ fhalf) << 4): the three terms occupy different bits
            // (pieces of a row: bits 4-6; rows: bits 7-14; stage offsets: multiples of 32 KB).
            // Weights ("deep" operand): three stages at 0, 32 KB, 64 KB; slots ("shallow"): two stages at 96 KB, 128 KB.
            constexpr uint32_t kShallowBase = 3 * 32768;
            static_assert(kTileBytes == 32768 && kTokTileBytes == 32768 && kRowBytes == 128, "address arithmetic above");
            typedef __attribute__((address_space(3))) const unsigned char* lds_ptr;
            const lds_ptr lds3 = (lds_ptr)lds;
            uint32_t base_w[kWF], base_t[kTF];
#pragma unroll
            for (int j = 0; j < kWF; ++j) base_w[j] = (uint32_t)(wrow[j] * kRowBytes + ((((wrow[j] >> 1) & 7) ^ fhalf) << 4));
#pragma unroll
            for (int i = 0; i < kTF; ++i) base_t[i] = (uint32_t)(trow[i] * kRowBytes + ((((trow[i] >> 1) & 7) ^ fhalf) << 4));
            constexpr int kL = kLoadsTok;       // loads per operand, wavefront and K step
            constexpr int kLB = kL / 2;         // of them per k16 block (an operand's loads go out over two blocks)
            static_assert(kLoadsPerOperand == kL && kL % 2 == 0, "issue slots below");
            bf16x8 tf[2][kTF], wf[2][kWF];
            const uint32_t wave_off = (uint32_t)(wave * kStageRows * kRowBytes);   // both operands: the same rows per wavefront
            auto dma_deep = [&](int stage, int kt, int q) {
                dma16(gp[kLoadsTok + q] + (size_t)kt * kRowBytes, lds0 + wave_off + (uint32_t)stage * 32768 + q * 1024);
            };
            auto dma_shallow = [&](int stage, int kt, int q) {
                dma16(gp[q] + (size_t)kt * kRowBytes,
                      lds0 + kShallowBase + wave_off + (uint32_t)stage * 32768 + q * 1024);
            };
            // In the first GEMM the main loop exists once per number of slot fragments with valid slots (TFE):
            // a wavefront of a ragged tile issues only the MFMAs and fragment reads of those (its loads stay
            // the same), finishes the tile sooner and the workgroup takes its next tile earlier.  persistent()
            // decides per launch whether that pays (`short_loops`).
            auto main_loop = [&](auto tfe_c) {
                constexpr int TFE = decltype(tfe_c)::value;
                constexpr int kM = kWF * TFE, kR = kWF + TFE;
                // One k16 block: the MFMAs of fragment buffer mbuf, between them the reads of k16 step rks of
                // the current stages into buffer rbuf, and loads at the MFMA slots the schedule names.
                auto block = [&](auto mfma, int mbuf, auto read, int rks, int rbuf, uint32_t w_off, uint32_t t_off, auto shallow,
                                 bool dma, int dstage, int dkt, int q0) {
#pragma unroll
                    for (int m = 0; m < (kM > kR ? kM : kR); ++m) {
                        if (decltype(mfma)::value && m < kM) {
                            const int i = m / kWF, j = m % kWF;
                            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[mbuf][j], tf[mbuf][i], acc[j][i], 0, 0, 0);
                        }
                        if (decltype(read)::value && m < kR) {
                            const uint32_t k_bits = (uint32_t)(rks << 5);
                            if (m < kWF)
                                wf[rbuf][m] = *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>(
                                    lds3 + (base_w[m] ^ (k_bits ^ w_off)));
                            else
                                tf[rbuf][m - kWF] = *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>(
                                    lds3 + (base_t[m - kWF] ^ (k_bits ^ t_off)));
                        }
                        // kLB loads per block, evenly spaced over its MFMAs
                        constexpr int kGap = kM / kLB;
                        static_assert(kM % kLB == 0, "issue slots");
                        if (dma && m < kM && m % kGap == kGap / 2) {
                            const int q = q0 + m / kGap;
                            if (decltype(shallow)::value) dma_shallow(dstage, dkt, q);
                            else dma_deep(dstage, dkt, q);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                };
                using Yes = std::true_type;
                using No = std::false_type;
                // prologue: deep operand of K steps 0 and 1 and shallow operand of K step 0, in the order the waits below assume
#pragma unroll
                for (int q = 0; q < kL; ++q) dma_deep(0, 0, q);
#pragma unroll
                for (int q = 0; q < kL; ++q) dma_shallow(0, 0, q);
                if (KT > 1) {
#pragma unroll
                    for (int q = 0; q < kL; ++q) dma_deep(1, 1, q);
                }
                int ds = 0, ss = 0;  // deep stage (kt % 3) and shallow stage (kt % 2) of the K step being computed
                for (int kt = 0; kt < KT; ++kt) {
                    // Outstanding, oldest first: deep operand of K step kt, shallow operand of K step kt, deep operand of
                    // K step kt + 1 (requested during K step kt - 1 after that K step's shallow loads); the last may stay in flight.
                    if (kt + 1 < KT) wait_vmcnt<kL>();
                    else wait_vmcnt<0>();
                    lds_barrier();
                    const uint32_t d_off = (uint32_t)ds * 32768, s_off = kShallowBase + (uint32_t)ss * 32768;
                    const uint32_t w_off = d_off, t_off = s_off;
                    const bool more_s = kt + 1 < KT, more_d = kt + 2 < KT;
                    const int ds2 = ds == 0 ? 2 : ds - 1;  // stage of K step kt + 2 = the one K step kt - 1 used
                    // last k16 step of K step kt - 1 (buffer 1) with the first reads of K step kt (buffer 0)
                    if (kt > 0) block(Yes{}, 1, Yes{}, 0, 0, w_off, t_off, Yes{}, more_s, ss ^ 1, kt + 1, 0);
                    else block(No{}, 1, Yes{}, 0, 0, w_off, t_off, Yes{}, more_s, ss ^ 1, kt + 1, 0);
                    block(Yes{}, 0, Yes{}, 1, 1, w_off, t_off, Yes{}, more_s, ss ^ 1, kt + 1, kLB);
                    block(Yes{}, 1, Yes{}, 2, 0, w_off, t_off, No{}, more_d, ds2, kt + 2, 0);
                    block(Yes{}, 0, Yes{}, 3, 1, w_off, t_off, No{}, more_d, ds2, kt + 2, kLB);
                    ds = ds == 2 ? 0 : ds + 1;
                    ss ^= 1;
                }
                block(Yes{}, 1, No{}, 0, 0, 0u, 0u, No{}, false, 0, 0, 0);
            };
            if constexpr (NMAT == 2) {
                switch (short_loops ? max(n_tf, 1) : kTF) {
                    case 1: main_loop(std::integral_constant<int, 1>{}); break;
                    case 2: main_loop(std::integral_constant<int, (kTF >= 2 ? 2 : kTF)>{}); break;
                    case 3: main_loop(std::integral_constant<int, (kTF >= 3 ? 3 : kTF)>{}); break;
                    default: main_loop(std::integral_constant<int, kTF>{}); break;
                }
            } else {
                main_loop(std::integral_constant<int, kTF>{});  // measured: the second GEMM is slower with the shorter loops
            }
        } else {
            // The loads of one stage are issued in kKSteps parts, one per k16 step of the K step being
            // computed, and within a k16 step one at a time between MFMAs (see step() below).
            // With only two stages the next K step is requested at once, in the first k16 step, so that it
            // has the whole K step to arrive; with a deeper ring the requests are spread over all k16 steps.
            constexpr int kM = kWF * kTF, kR = kWF + kTF;
            constexpr int kDmaParts = STAGES == 2 ? (kLoads <= kM ? 1 : 2) : (kLoads % kKSteps == 0 ? kKSteps : 2);
            static_assert(kLoads % kDmaParts == 0, "loads per stage must split evenly over the k16 steps that issue them");
            constexpr int kLoadsPerPart = kLoads / kDmaParts;
            // SKIP: a wavefront whose 32 slot rows all lie past the tile's last slot stages no slot rows (the
            // fragments they would feed are skipped as well): a ragged tile then moves its weights plus only
            // its own slot rows through the load path, which is what bounds tiles of cold experts.
            static_assert(!SKIP || 32 % kTokStageRows == 0, "a wavefront stages rows of one 32-slot fragment");
            const bool stage_tok = !SKIP || (wave * kTokStageRows) / 32 * 32 < rows;  // its fragment has valid slots
            auto dma_one = [&](int stage, int kt, int l) {
                if (SKIP && l < kLoadsTok && !stage_tok) return;
                const uint32_t base = lds0 + (uint32_t)stage * kStageBytes;
                dma16(gp[l] + (size_t)kt * kRowBytes,
                      base + (l < kLoadsTok ? stage_off_tok + l * 1024 : stage_off_w + (l - kLoadsTok) * 1024));
            };

            // Operand fragments are double-buffered in registers (buffer = k16 step & 1).  One pipeline
            // step issues the MFMAs of one k16 step and, BETWEEN them one for one, the LDS reads of the
            // next step's fragments (into the other buffer) and this wavefront's share of the global->LDS
            // loads of a later K step.  Interleaving matters: a burst of ds_reads from all wavefronts right
            // after a barrier fills the LDS command queue and blocks the issuing wavefronts, MFMAs
            // included; one read per MFMA keeps the matrix pipe fed while the queue drains.  The MFMAs of a
            // K step's LAST k16 step run after the next K step's barrier, paired with its first reads, so
            // the matrix pipe also has work while the wavefronts re-synchronise.
            static_assert(kKSteps % 2 == 0, "fragment buffers alternate per k16 step");
            static_assert(kLoadsPerPart <= kM, "a step has one slot per MFMA for its loads");
            bf16x8 tf[2][kTF], wf[2][kWF];
            auto read_one = [&](int stage, int ks, int buf, int idx) {
                const unsigned char* st = lds + stage * kStageBytes;
                if (idx < kWF)
                    wf[buf][idx] = *reinterpret_cast<const bf16x8*>(
                        st + kTokTileBytes + wrow[idx] * kRowBytes + (Swz<BK>::piece(wrow[idx], ks * 2 + fhalf) << 4));
                else if (!SKIP || idx - kWF < n_tf)
                    tf[buf][idx - kWF] = *reinterpret_cast<const bf16x8*>(
                        st + trow[idx - kWF] * kRowBytes + (Swz<BK>::piece(trow[idx - kWF], ks * 2 + fhalf) << 4));
            };
            // mfma: issue the MFMAs of buffer mbuf.  read: fetch fragments (rstage, rks) into buffer rbuf.
            // dma: issue part dpart of K step dkt's loads into stage dstage.
            auto step = [&](auto mfma, int mbuf, auto read, int rstage, int rks, int rbuf, bool dma, int dstage, int dkt,
                            int dpart) {
    #pragma unroll
                for (int m = 0; m < kM; ++m) {
                    if (decltype(mfma)::value) {
                        const int i = m / kWF, j = m % kWF;
                        if (!SKIP || i < n_tf)
                            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[mbuf][j], tf[mbuf][i], acc[j][i], 0, 0, 0);
                    }
                    if (decltype(read)::value && m < kR) read_one(rstage, rks, rbuf, m);
                    if (m >= kM - kLoadsPerPart && dma && dpart < kDmaParts)
                        dma_one(dstage, dkt, dpart * kLoadsPerPart + m - (kM - kLoadsPerPart));
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            using Yes = std::true_type;
            using No = std::false_type;

            // prologue: STAGES - 1 K steps in flight
    #pragma unroll
            for (int s = 0; s < STAGES - 1; ++s)
                if (s < KT) {
    #pragma unroll
                    for (int l = 0; l < kLoads; ++l) dma_one(s, s, l);
                }
            for (int kt0 = 0; kt0 < KT; kt0 += STAGES) {
    #pragma unroll
                for (int s = 0; s < STAGES; ++s) {
                    const int kt = kt0 + s;
                    if (kt < KT) {
                        // K step kt must have landed; up to STAGES - 2 younger ones may stay in flight
                        if (kt + STAGES - 2 >= KT) wait_vmcnt<0>();
                        else if (stage_tok) wait_vmcnt<(STAGES - 2) * kLoads>();
                        else wait_vmcnt<(STAGES - 2) * kLoadsPerOperand>();  // this wavefront issues weight loads only
                        lds_barrier();
                        const bool more = kt + STAGES - 1 < KT;
                        const int ns = (s + STAGES - 1) % STAGES;
                        // last k16 step of K step kt - 1 (buffer 1) with the first reads of K step kt (buffer 0)
                        if (kt > 0) step(Yes{}, 1, Yes{}, s, 0, 0, more, ns, kt + STAGES - 1, 0);
                        else step(No{}, 1, Yes{}, s, 0, 0, more, ns, kt + STAGES - 1, 0);
    #pragma unroll
                        for (int ks = 0; ks + 1 < kKSteps; ++ks)
                            step(Yes{}, ks & 1, Yes{}, s, ks + 1, (ks + 1) & 1, more, ns, kt + STAGES - 1, ks + 1);
                    }
                }
            }
            step(Yes{}, (kKSteps - 1) & 1, No{}, 0, 0, 0, false, 0, 0, kDmaParts);
        }

        // Ask for the next work item now; the answer is needed only after the epilogue.
        int next_item = 0;
        if (tid == 0) next_item = __hip_atomic_fetch_add(handed_out, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // ---- split tiles: publish this piece; the last piece to arrive sums them all in part order.
        bool finish = true;  // this workgroup writes the tile's result
        if (parts > 1) {
            float* mine = partials + (size_t)part * kPartialFloats;
            // The stores below are issued from inline asm, which the compiler's hazard bookkeeping does
            // not cover: leave the last MFMAs time to write their results (19 wait states at most).
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
            for (int j = 0; j < kWF; ++j)
#pragma unroll
                for (int i = 0; i < kTF; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        f32x4 v;
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = acc[j][i][q * 4 + c];
                        store16_through(mine + ((size_t)((j * kTF + i) * 4 + q) * kThreads + tid) * 4, v);
                    }
            // The pieces are written through to memory (device-scope stores), so once every wavefront's
            // stores have been acknowledged (vmcnt 0, then the barrier) one relaxed atomic can count the
            // arrival: no cache has to be written back.  Only the workgroup that sums the pieces
            // invalidates its caches before it reads them.  (An acquire-release atomic per arrival
            // would add an L2 write-back each time, tens of microseconds in all.)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            int* flag = reinterpret_cast<int*>(lds);
            if (tid == 0) *flag = __hip_atomic_fetch_add(arrivals, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            finish = __builtin_amdgcn_readfirstlane(*flag) == parts - 1;
            __syncthreads();  // everyone has read the flag before LDS is reused
        }
        if (finish && parts > 1) {
            // one wavefront drops whatever this CU's cache may hold of the pieces (an invalidate, no write-back)
            if (tid == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            __syncthreads();
#pragma unroll
            for (int j = 0; j < kWF; ++j)
#pragma unroll
                for (int i = 0; i < kTF; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;
            for (int p = 0; p < parts; ++p) {
                const float* src = partials + (size_t)p * kPartialFloats;
#pragma unroll
                for (int j = 0; j < kWF; ++j)
#pragma unroll
                    for (int i = 0; i < kTF; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 v =
                                *reinterpret_cast<const f32x4*>(src + ((size_t)((j * kTF + i) * 4 + q) * kThreads + tid) * 4);
#pragma unroll
                            for (int c = 0; c < 4; ++c) acc[j][i][q * 4 + c] += v[c];
                        }
            }
        }

        // ---- epilogue: transpose through LDS so that global stores are whole contiguous rows.
        // MFMA 32x32 result: lane holds column (slot) lane & 31 and rows (weight rows)
        // 8 * (r / 4) + 4 * (lane / 32) + (r % 4), r = 0..15, i.e. 4 consecutive features per r / 4.
        // LDS rows are XOR-swizzled in 16-byte units so the row-wise read-back is conflict free.
        lds_barrier();  // every wavefront is done reading operand tiles; no load is outstanding
        if (!finish) {
            // another workgroup sums this tile's pieces
        } else if (NMAT == 2) {
            // [256 slots][128 features] bf16, 256-byte rows, unit v of row r at position v ^ (r & 15)
#pragma unroll
            for (int i = 0; i < kTF; ++i) {
                const int row = (i * WT + wt) * 32 + frow;
#pragma unroll
                for (int jf = 0; jf < kFragsPerMat; ++jf) {
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int col = wq * kFeatPerWave + jf * 32 + rg * 8 + fhalf * 4;  // feature in tile
                        float o[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            o[c] = swiglu(acc[jf][i][rg * 4 + c], acc[kFragsPerMat * (NMAT - 1) + jf][i][rg * 4 + c]);
                        uint2 pk;
                        pk.x = pack_bf16x2(o[0], o[1]);
                        pk.y = pack_bf16x2(o[2], o[3]);
                        const int unit = col >> 3;
                        *reinterpret_cast<uint2*>(lds + row * 256 + ((unit ^ (row & 15)) << 4) + (col & 4) * 2) = pk;
                    }
                }
            }
            lds_barrier();
            for (int row = tid >> 4; row < rows; row += kThreads / 16) {
                const int unit = tid & 15;
                const int n = n0 + unit * 8;
                if (n < N) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * 256 + ((unit ^ (row & 15)) << 4));
                    *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(dst) + (size_t)(slot0 + row) * N + n) = v;
                }
            }
        } else {
            // per slot frag i: [32 * WT slots][256 features] fp32, 1 KB rows, unit v of row r at v ^ (r & 63)
#pragma unroll
            for (int i = 0; i < kTF; ++i) {
                if (i > 0) lds_barrier();
                const int lrow_e = wt * 32 + frow;
#pragma unroll
                for (int jf = 0; jf < kFragsPerMat; ++jf) {
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int unit = (wq * kFeatPerWave + jf * 32 + rg * 8 + fhalf * 4) >> 2;
                        f32x4 v;
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = acc[jf][i][rg * 4 + c];
                        *reinterpret_cast<f32x4*>(lds + lrow_e * 1024 + ((unit ^ (lrow_e & 63)) << 4)) = v;
                    }
                }
                lds_barrier();
                for (int lr = wave; lr < 32 * WT; lr += kWaves) {
                    const int row = i * (32 * WT) + lr;  // slot in tile: fragment i * WT + lr / 32
                    const int n = n0 + lane * 4;
                    if (row < rows && n < N) {
                        const f32x4 v = *reinterpret_cast<const f32x4*>(lds + lr * 1024 + ((lane ^ (lr & 63)) << 4));
                        *reinterpret_cast<f32x4*>(static_cast<float*>(dst) + (size_t)(slot0 + row) * N + n) = v;
                    }
                }
            }
        }
        // ---- hand the next item's number to every wavefront.  The first barrier also keeps the next
        // tile's loads from landing in LDS that a slower wavefront is still reading back above; the word
        // sits in the stage that no load is written to before the next tile's first barrier.
        lds_barrier();
        int* handoff = reinterpret_cast<int*>(lds + kHandoffOffset);
        if (tid == 0) *handoff = next_item;
        lds_barrier();
        return __builtin_amdgcn_readfirstlane(*handoff);
    }
};

template <int NMAT, int BK, int STAGES, int WT, int WW, bool SKIP, int BT = kBT, bool W3 = false>
__global__ __launch_bounds__(WT * WW * 64, 1) void grouped_gemm_kernel(const uint16_t* __restrict__ tok_base,
                                                                    const uint16_t* __restrict__ wa,
                                                                    const uint16_t* __restrict__ wb,
                                                                    const int32_t* __restrict__ offs,
                                                                    const int32_t* __restrict__ row_of_slot, int E,
                                                                    int topk, int N, int K, void* __restrict__ dst,
                                                                    int32_t* __restrict__ sync,
                                                                    float* __restrict__ scratch) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_dyn[];
    Gemm<NMAT, BK, STAGES, WT, WW, SKIP, BT, false, W3>::persistent(tok_base, wa, wb, offs, row_of_slot, E, topk, N, K, dst,
                                                                    sync, scratch, lds_dyn);
}

// gemm1 with per-selection input rows (see Gemm's ALT).
template <int BK, int STAGES, int WT, int WW, bool SKIP, int BT = kBT, bool W3 = false>
__global__ __launch_bounds__(WT * WW * 64, 1) void grouped_gemm1_alt_kernel(
    const uint16_t* __restrict__ tok_base, const uint16_t* __restrict__ tok_alt, const uint8_t* __restrict__ alt_mask,
    const uint16_t* __restrict__ wa, const uint16_t* __restrict__ wb, const int32_t* __restrict__ offs,
    const int32_t* __restrict__ row_of_slot, int E, int topk, int N, int K, void* __restrict__ dst,
    int32_t* __restrict__ sync, float* __restrict__ scratch) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds_dyn[];
    Gemm<2, BK, STAGES, WT, WW, SKIP, BT, true, W3>::persistent(tok_base, wa, wb, offs, row_of_slot, E, topk, N, K, dst, sync,
                                                            scratch, lds_dyn, tok_alt, alt_mask);
}

}  // namespace gg
}  // namespace moe
