// The MoE layer for decode-size calls (a handful of tokens), bf16 storage, as
// ONE persistent kernel: routing, both expert GEMMs and the weighted combine.
//
// With the experts resident in HBM, a decode step of the MoE layer is a weight
// stream: each selected expert's three matrices are read once and multiplied
// by a few hidden states (the paper's Table I discussion: expert parameters
// dwarf the activations by four orders of magnitude).  At one token the stream
// lasts little more than 100 microseconds, so every kernel boundary, cold
// start and dependent memory latency is a visible fraction of the layer.  The
// kernel is therefore organised around the HBM stream, not around the
// arithmetic:
//
//   * every workgroup evaluates the gate for all tokens itself (the gate is
//     64-128 KB and the arithmetic is the same everywhere, so all workgroups
//     agree bit for bit); workgroup 0 publishes indices, weights and counts;
//   * no token permutation and no LDS staging of weights: every weight byte is
//     used by exactly one wavefront, so it is loaded straight into registers
//     with 16-byte loads, consecutive lanes on consecutive addresses;
//   * every load instruction covers 8 weight rows x 128 contiguous bytes (whole
//     cache lines; 64-byte pieces stream measurably slower).  The natural
//     operand layout of v_mfma_f32_16x16x32_bf16 would give 16 rows x 64 bytes,
//     so the 16 operand rows are used as 8 weight rows x 2 halves of a 64-wide
//     K step instead: a second load fetches the next 8 weight rows, a cross-lane
//     rearrangement and a per-lane select recombine the two loads into one
//     operand holding the lower K half of all 16 weight rows and one holding
//     the upper half (with rows i and i ^ 8 exchanged), and two MFMAs with the
//     matching halves of the tokens accumulate them; the two accumulators are
//     added, after undoing the row exchange with a cross-lane move, when the
//     tile is finished;
//   * the tokens of an expert form the 16 columns of the MFMA, so up to 16
//     tokens share one pass over the weights;
//   * every load of the streaming loops is unconditional (steps, tiles and token
//     columns that do not exist re-read a valid address and are multiplied by
//     zeros or ignored), so the compiler can count outstanding loads and wait
//     for exactly the step it needs;
//   * each wavefront keeps P steps of loads in flight in a rotating register
//     window (software pipeline unrolled P times) that runs across tile and
//     expert boundaries, and the barrier at a tile's end waits for LDS only, so
//     the stream never drains.  With 2048 wavefronts on the chip a shallow
//     window is enough and measurably better than a deep one (P = 1 for the
//     first GEMM, 2 for the second; 4 and 8 lose 2-3 %);
//   * the 8 wavefronts of a workgroup split K (interleaved 64-element steps),
//     and their partial 16 x 16 tiles are summed through LDS in a fixed order
//     (deterministic);
//   * between the two GEMMs every workgroup needs the whole intermediate
//     vector of an expert before it multiplies by that expert's W2: a
//     grid-wide rendezvous made of one arrival flag per workgroup, each set to
//     a per-launch epoch, so the flags never need clearing and no
//     read-modify-write atomic is contended.  The experts are taken in two
//     groups with a rendezvous each (see announce()), which the workgroups
//     reach long after the others have passed, so nobody waits for the slowest
//     workgroup in the middle of the call.  The intermediate is written with
//     device-scope (write-through) stores, so it has reached memory when the
//     flag is raised, and it is read with ordinary loads only after the
//     rendezvous: no L2 holds an older copy, because caches are invalidated
//     when a kernel starts and nothing reads a group's intermediate before its
//     rendezvous.  This keeps the rendezvous free of cache write-backs and
//     invalidations (a device-scope fence issued by every wavefront of the grid
//     costs tens of microseconds here).  The first P steps of the second GEMM's
//     weights are requested before the first rendezvous is awaited, so the
//     stream continues across it.
//
//   phase 1: act[a, f] = silu(x[t] . w1[e, f]) * (x[t] . w3[e, f])   a = t*k + j, e = idx[a]
//   phase 2: y[t, h]   = sum over the token's experts (ascending expert id) of
//                        w[a] * (act[a] . w2[e, h]),  fp32, one rounding to bf16
#include "bf16_utils.h"
#include "moe_internal.h"
#include "route_device.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Pipeline depths (64-element K steps of loads in flight per wavefront) of the two GEMM phases.
constexpr int kP1 = 1, kP2 = 2;

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
// How the 8 wavefronts of a workgroup split K: interleaved 64-element steps (wavefront w takes steps
// w, w + 8, ...), so that at any moment the workgroup reads one contiguous 1 KB piece of each weight row.
struct KSplit {
    int n_valid;     // steps of this wavefront
    int stride;      // elements between its consecutive steps
    size_t k0;       // element offset of its first step
    int per;         // steps of the busiest wavefront
    __device__ KSplit(int k_steps, int wave) {
        per = (k_steps + kWaves - 1) / kWaves;
        n_valid = wave < k_steps ? (k_steps - wave + kWaves - 1) / kWaves : 0;
        stride = 64 * kWaves;
        k0 = (size_t)wave * 64;
    }
};
// An expert's tokens are the columns of 16x16x32 MFMAs: NC column groups of 16 serve calls of up to
// 16 * NC tokens (a token selects an expert at most once, so no expert sees more tokens than the call has).
static_assert(kStreamMaxTokens == 32, "column groups are instantiated for 16 and 32 tokens");
static_assert(kThreads == kSmallRouteThreads && kDecodeMaxTokens == kSmallRouteMaxTokens,
              "in-kernel routing runs in the same workgroup");

struct DecodeArgs {
    const uint16_t* x;      // [T, H]
    // routing: either a gate to evaluate (wg != null; idx_out / w_out / counts are written by
    // workgroup 0) or selections made earlier (idx_in / w_in)
    const uint16_t* wg;
    const float* bias;
    int32_t* idx_out;
    float* w_out;
    int32_t* counts;
    int accumulate;
    const int32_t* idx_in;
    const float* w_in;
    // prediction with the next layer's gate (wg_next may be null): pred_out [T, k]
    const uint16_t* wg_next;
    const float* bias_next;
    int32_t* pred_out;
    // pre-calculated selections (ALT kernels only): assignment a reads x_stale instead of x when stale[a] != 0
    const uint16_t* x_stale;
    const uint8_t* stale;
    const uint16_t *w1, *w3, *w2;
    uint16_t* act;          // [T*k, F] workspace
    uint16_t* y;            // [T, H]
    uint32_t* flags;        // workspace: 2 x kFlagStride arrival flags of the two rendezvous, then the epoch word
                            // and the status word (see kStatusIndex)
    int spin_limit;         // polling rounds a rendezvous waits before it gives up
    int T, k, E, H, F;
};

template <int NC>
struct Groups {
    static constexpr int kMaxTok = 16 * NC;
    int n_active;
    int expert[64];           // active experts, ascending id
    int cnt[64];              // tokens of that expert (<= 16 * NC)
    int assign[64][kMaxTok];  // their assignment ids t*k + j, ascending
};

// Builds the per-expert token lists from the selections in LDS; call with all threads, ends with
// a barrier.
template <int NC>
__device__ void build_groups(Groups<NC>& g, const int* idx, int A, int E) {
    constexpr int kMaxTok = Groups<NC>::kMaxTok;
    const int tid = threadIdx.x;
    if (tid < 64) {
        int c = 0;
        if (tid < E) {
            for (int a = 0; a < A; ++a) {
                const int e = min(max(idx[a], 0), E - 1);
                if (e == tid && c < kMaxTok) ++c;
            }
        }
        const uint64_t present = __ballot(c > 0);
        const int ord = __popcll(present & ((1ull << tid) - 1ull));
        if (tid == 0) g.n_active = __popcll(present);
        if (c > 0) {
            g.expert[ord] = tid;
            g.cnt[ord] = c;
            int n = 0;
            for (int a = 0; a < A; ++a) {
                const int e = min(max(idx[a], 0), E - 1);
                if (e == tid && n < kMaxTok) g.assign[ord][n++] = a;
            }
        }
    }
    __syncthreads();
}

// Every load of the streaming loops is unconditional: a load under a branch cannot be counted by
// the compiler, which then waits for ALL outstanding loads before each use (s_waitcnt vmcnt(0)) and
// the software pipeline degenerates into "request P steps, wait for all of them".  Steps, tiles and
// token columns that do not exist therefore re-read a valid address of the same operand (a cache
// hit), and their contribution is removed by zeroing the token operand when it is used.
__device__ inline u32x4 load16(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

__device__ inline u32x4 keep_if(bool on, u32x4 v) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = on ? v[i] : 0u;
    return r;
}

__device__ inline bf16x8 pick(bool first, u32x4 a, u32x4 b) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = first ? a[i] : b[i];
    return __builtin_bit_cast(bf16x8, v);
}

// Barrier that orders LDS traffic only: loads from global memory stay in flight across it.
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- grid-wide rendezvous between the two GEMMs, in two stages.
// The active experts are split into a first group (the lower half of the ascending list, group A)
// and the rest (group B).  Phase 1 visits a workgroup's tiles in expert order, phase 2 its experts
// in the same order, so a workgroup raises flag A when it has stored its last intermediate values
// of group A, goes on with group B, raises flag B, and in phase 2 needs everybody's flag A only
// before its first group-A operand and everybody's flag B only before its first group-B operand.
// By then the others have normally been past that point for tens of microseconds, so nobody
// waits for the slowest workgroup between the phases (a single rendezvous costs the mean
// workgroup about 6 us of a 128 us call: the spread of the phase-1 finishing times).
// A flag is "raised" when it holds the launch's epoch; the two flag arrays are kFlagStride apart.
constexpr int kFlagStride = 256;
// The epoch is a launch count kept in the workspace too (one word after the flags): a launch reads
// it when it starts and uses count + 1; workgroup 0 stores the new count when it ends, by which time
// every workgroup has read the old one (workgroup 0 has passed a rendezvous that all of them had to
// reach).  Flags left by earlier launches carry earlier epochs, and arbitrary memory contents equal
// the new epoch only by accident, so nothing ever needs clearing; and because no launch argument
// changes from call to call, a call recorded into a HIP graph can be replayed.
constexpr int kEpochIndex = 2 * kFlagStride;
// The word after the epoch reports a rendezvous that gave up (its bounded wait ran out because the
// grid was not resident all at once): the workgroup stores kDecodeGaveUp there and writes NaN
// instead of its output tiles.  Nothing else ever writes the word, so it stays set until the host
// resets it (moe_decode_status).
constexpr int kStatusIndex = kDecodeStatusWord;
static_assert(kStatusIndex == kEpochIndex + 1 && kStatusIndex < kDecodeFlagInts, "flags, epoch and status fit the workspace block");

// All of this workgroup's stores to `act` so far have left the CU; then raise `flag`.
__device__ inline void announce(uint32_t* flag, uint32_t epoch) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits (all threads) until the n flags all hold `epoch`.  The spin is bounded (`limit` polling
// rounds), so the kernel ends even if the workgroups never become co-resident; a wait that runs out
// marks the call as failed: the status word in the workspace and *failed (LDS, read when y is stored).
// Global loads already in flight stay in flight.
__device__ inline void await_flags(const uint32_t* flags, int n, uint32_t epoch, int limit, uint32_t* status,
                                   int* failed) {
    if (threadIdx.x < 64) {
        bool met = false;
        for (int it = 0; it < limit; ++it) {
            bool all = true;
            for (int i = threadIdx.x; i < n; i += 64)
                all &= __hip_atomic_load(&flags[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == epoch;
            if (__all(all)) {
                met = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!met && threadIdx.x == 0) {
            __hip_atomic_store(status, kDecodeGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *failed = 1;
        }
    }
    asm volatile("" ::: "memory");
    lds_barrier();
    asm volatile("" ::: "memory");  // no load of `act` may be moved above the rendezvous
}

// acc1 holds MFMA row i = weight row i, acc2 holds MFMA row i = weight row i ^ 8; MFMA rows
// 4 * (lane / 16) + r sit in lane, so row i ^ 8 is the same register of lane ^ 32.
__device__ inline f32x4 fold_halves(f32x4 acc1, f32x4 acc2) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = acc1[i] + __shfl_xor(acc2[i], 32, 64);
    return r;
}

// Per-lane element offsets inside a tile of 16 weight rows and a 64-element K step.
//
// Loads are issued with consecutive lanes on consecutive addresses: lane s reads the 16-byte piece
// s % 8 of row s / 8 (8 rows x 128 contiguous bytes per instruction).  The MFMA wants row
// lane % 16 and K group lane / 16 in each lane, which scatters the lanes of every quad over four
// rows; loading in that order costs the address path four cache-line lookups where one would do
// (measured: an isolated tile takes 3.4 times as long, the saturated stream 3-4 % longer).  So the
// loaded registers are rearranged across lanes afterwards (ds_bpermute, no LDS memory involved):
// MFMA lane l = (i = l % 16, kq = l / 16) takes, from the load of rows 0-7, row i % 8 and piece
// (i >= 8 ? 4 : 0) + kq, and from the load of rows 8-15, row 8 + i % 8 and piece (i >= 8 ? 0 : 4) + kq
// (the two K halves swapped), which is the pair of layouts mfma_operands() recombines.
struct LaneMap {
    int row_lo, row_hi;    // weight rows (within the tile) this lane loads in the two loads
    int k_ld;              // element offset of the 8 elements it loads inside the K step
    int perm_lo, perm_hi;  // byte index (4 * source lane) for ds_bpermute after the two loads
    int kq8;               // element offset of the lane's token operand inside each 32-element half
    bool upper;
    __device__ explicit LaneMap(int lane) {
        const int i = lane & 15, kq = lane >> 4;
        upper = i >= 8;
        row_lo = lane >> 3;
        row_hi = 8 + (lane >> 3);
        k_ld = (lane & 7) * 8;
        perm_lo = ((i & 7) * 8 + (upper ? 4 : 0) + kq) * 4;
        perm_hi = ((i & 7) * 8 + (upper ? 0 : 4) + kq) * 4;
        kq8 = kq * 8;
    }
};

__device__ inline u32x4 gather_lanes(int byte_index, u32x4 v) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(byte_index, (int)v[i]);
    return r;
}

// From the raw loads of rows 0-7 and rows 8-15 of a K step: `first` holds the lower K half of all
// 16 weight rows (MFMA row i = weight row i), `second` the upper half with rows i and i ^ 8 exchanged.
__device__ inline void mfma_operands(const LaneMap& lm, u32x4 lo_raw, u32x4 hi_raw, bf16x8& first, bf16x8& second) {
    const u32x4 lo = gather_lanes(lm.perm_lo, lo_raw), hi = gather_lanes(lm.perm_hi, hi_raw);
    first = pick(lm.upper, hi, lo);
    second = pick(lm.upper, lo, hi);
}

template <int NC>
struct Smem {
    int idx[16 * NC * 8];     // selections of the call (expert per assignment) ...
    float w[16 * NC * 8];     // ... and their weights
    RouteSmem route;          // scratch of the in-kernel routing (NC == 1 only)
    Groups<NC> g;
    // partial tiles of the 8 wavefronts; double-buffered over consecutive tiles while that fits
    static constexpr int kRedBufs = NC >= 4 ? 1 : 2;
    f32x4 red[kRedBufs][kWaves][2][NC][64];
    float yacc[16 * NC][16];
    int failed;               // a rendezvous of this workgroup gave up: its output tiles become NaN
    unsigned char stale[16 * NC * 8];  // ALT kernels: the call's stale mask, per assignment
};

// ---- phase 1: act[a, f] = silu(x[t] . w1[e, f]) * (x[t] . w3[e, f]) over this workgroup's share
// of the (active expert, 16-feature tile) list.
// Row of the token operand of assignment a: x, or x_stale for a pre-calculated selection (ALT).
template <bool ALT, int NC>
__device__ inline const uint16_t* token_row(const DecodeArgs& p, const Smem<NC>& sm, int a) {
    const uint16_t* base = (ALT && sm.stale[a] != 0) ? p.x_stale : p.x;
    return base + (size_t)(a / p.k) * p.H;
}

template <int P, int NC, bool ALT>
__device__ inline void gemm1_phase(const DecodeArgs& p, Smem<NC>& sm, uint32_t epoch, bool& a_open) {
    const Groups<NC>& g = sm.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15;
    const LaneMap lm(lane);
    const int H = p.H, F = p.F, k = p.k;

    const int tiles_per_expert = F / 16;
    const int total_tiles = g.n_active * tiles_per_expert;
    const int tiles_per_wg = (total_tiles + gridDim.x - 1) / gridDim.x;
    const int t0 = blockIdx.x * tiles_per_wg;
    const int t1 = min(total_tiles, t0 + tiles_per_wg);
    if (t0 >= t1) return;

    // K split: 64-element steps dealt to the wavefronts in contiguous runs.
    const KSplit ks(H / 64, wave);
    const int n_valid = ks.n_valid, kstride = ks.stride;
    const int spt = (ks.per + P - 1) / P * P;  // steps per tile, padded to the pipeline depth
    const long total_q = (long)(t1 - t0) * spt;
    const size_t k0 = n_valid > 0 ? ks.k0 : 0;  // a wavefront without steps re-reads the row's start

    u32x4 lo1[P], hi1[P], lo3[P], hi3[P], xa[P][NC], xb[P][NC];
    // Issue-side state: the next step to request and the row bases of its tile.
    int is = 0, itile = t0;
    size_t wlo = 0, whi = 0;
    const uint16_t* xbase[NC];
    auto enter_tile = [&]() {
        const int d = itile / tiles_per_expert;
        const int f0 = (itile - d * tiles_per_expert) * 16;
        const size_t row0 = (size_t)g.expert[d] * F + f0;
        wlo = (row0 + lm.row_lo) * H + k0 + lm.k_ld;
        whi = (row0 + lm.row_hi) * H + k0 + lm.k_ld;
#pragma unroll
        for (int c = 0; c < NC; ++c)  // columns without a token read the expert's first token (result unused)
            xbase[c] = token_row<ALT, NC>(p, sm, g.assign[d][col + 16 * c < g.cnt[d] ? col + 16 * c : 0]) + k0 + lm.kq8;
    };
    enter_tile();
    auto issue = [&](int i) {  // requests past the last tile re-read it
        const size_t off = (size_t)(is < n_valid ? is : 0) * kstride;
        lo1[i] = load16(p.w1 + wlo + off);
        hi1[i] = load16(p.w1 + whi + off);
        lo3[i] = load16(p.w3 + wlo + off);
        hi3[i] = load16(p.w3 + whi + off);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            xa[i][c] = load16(xbase[c] + off);
            xb[i][c] = load16(xbase[c] + off + 32);
        }
        if (++is == spt) {
            is = 0;
            if (++itile < t1) enter_tile();
        }
    };
#pragma unroll
    for (int i = 0; i < P; ++i) issue(i);  // total_q >= spt >= P

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 g1[NC], g2[NC], u1[NC], u2[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) g1[c] = g2[c] = u1[c] = u2[c] = zero;
    const int d_a = (g.n_active + 1) / 2;  // experts [0, d_a) of the active list are group A
    int cs = 0, ctile = t0;
    for (long q = 0; q < total_q; q += P) {
        if (a_open && cs == 0 && ctile / tiles_per_expert >= d_a) {  // group A is complete here
            announce(&p.flags[blockIdx.x], epoch);
            a_open = false;
        }
#pragma unroll
        for (int i = 0; i < P; ++i) {
            bf16x8 a1, a2, a3, a4;
            mfma_operands(lm, lo1[i], hi1[i], a1, a2);
            mfma_operands(lm, lo3[i], hi3[i], a3, a4);
            const bool real = cs + i < n_valid;  // a padding step multiplies zeros
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const bf16x8 b1 = __builtin_bit_cast(bf16x8, keep_if(real, xa[i][c]));
                const bf16x8 b2 = __builtin_bit_cast(bf16x8, keep_if(real, xb[i][c]));
                g1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1, g1[c], 0, 0, 0);
                g2[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b2, g2[c], 0, 0, 0);
                u1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b1, u1[c], 0, 0, 0);
                u2[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a4, b2, u2[c], 0, 0, 0);
            }
            issue(i);
        }
        cs += P;
        if (cs == spt) {
            // Tile done: fold the 8 K-slices.  MFMA 16x16 result: lane holds column (token)
            // lane & 15 and rows (features) 4 * (lane / 16) + r, r = 0..3.
            const int par = (ctile - t0) % Smem<NC>::kRedBufs;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                sm.red[par][wave][0][c][lane] = fold_halves(g1[c], g2[c]);
                sm.red[par][wave][1][c][lane] = fold_halves(u1[c], u2[c]);
            }
            lds_barrier();
            const int d = ctile / tiles_per_expert;
            const int f0 = (ctile - d * tiles_per_expert) * 16;
            const int cnt = g.cnt[d];
            // one reducer per (column group, lane, feature pair): 128 * NC work items
            for (int item = tid; item < 128 * NC; item += kThreads) {
                const int c = item >> 7, pl = item & 63, rp = (item >> 6) & 1;
                const int tok = (pl & 15) + 16 * c;
                if (tok < cnt) {
                    float o[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        float gs = 0.f, us = 0.f;
#pragma unroll
                        for (int w = 0; w < kWaves; ++w) {
                            gs += sm.red[par][w][0][c][pl][2 * rp + h];
                            us += sm.red[par][w][1][c][pl][2 * rp + h];
                        }
                        o[h] = swiglu(gs, us);
                    }
                    // device-scope (write-through) store: read by other workgroups after the grid barrier
                    uint32_t* dst = reinterpret_cast<uint32_t*>(p.act + (size_t)g.assign[d][tok] * F + f0 +
                                                                4 * (pl >> 4) + 2 * rp);
                    __hip_atomic_store(dst, pack_bf16x2(o[0], o[1]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            if (Smem<NC>::kRedBufs == 1) lds_barrier();  // the single buffer is free again
#pragma unroll
            for (int c = 0; c < NC; ++c) g1[c] = g2[c] = u1[c] = u2[c] = zero;
            cs = 0;
            ++ctile;
        }
    }
}

// ---- phase 1 when a wavefront's K slice is at most kXSteps steps (hidden <= 4096): the token
// operand of an expert is the same for every feature tile, so its fragments are loaded once per
// expert and stay in registers; only weights stream.  A tile is exactly kXSteps steps (statically
// indexed fragments), steps past the slice multiply zeros.
//
// Tiles are dealt to the workgroups round-robin (tile b + n * grid), so every XCD reads from every
// part of the matrices.  (How fast a workgroup streams depends on where its data lives relative to
// its XCD, by several percent and differently in every call.  Handing the last rounds out on demand
// from ticket counters was measured and lost: a unit has to be claimed a unit or two ahead to keep
// the load pipeline full, which is as coarse as the imbalance it is meant to remove, and the
// counters cost more than they saved.)
constexpr int kXSteps = 8;
// Workgroups that take part in phase 1: as many as are needed for the busiest one's tile count,
// ceil(tiles / ceil(tiles / grid)); 800 tiles go to 200 workgroups with 4 each rather than to 256
// with 3 or 4.  The HBM stream is the shared resource, so a balanced share over fewer workgroups
// ends when the bytes are through, while an unbalanced one ends with a few workgroups streaming
// alone at their latency-bound rate (800-tile case: phase 1 ends at 44 instead of 47 us; a deeper
// load window for the fewer streams did not help further).
__device__ inline int phase1_participants(int total_tiles, int grid) {
    const int busiest = (total_tiles + grid - 1) / grid;
    return (total_tiles + busiest - 1) / max(busiest, 1);
}
template <int P, int NC, bool ALT>
__device__ inline void gemm1_phase_xreg(const DecodeArgs& p, Smem<NC>& sm, uint32_t epoch, bool& a_open) {
    static_assert(kXSteps % P == 0, "the weight ring must divide a tile");
    const Groups<NC>& g = sm.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15;
    const LaneMap lm(lane);
    const int H = p.H, F = p.F, k = p.k;

    const int tiles_per_expert = F / 16;
    const int total_tiles = g.n_active * tiles_per_expert;
    // This workgroup's tiles, numbered n = 0 .. n_mine - 1 in ascending tile order.
    // Only as many workgroups take part as are needed for the busiest one's tile count (see
    // phase1_participants()).
    // Round n deals tiles [n * g1, (n + 1) * g1) to the participants rotated by n * kRot, so that a
    // workgroup (and with it an XCD, which owns every 8th workgroup) does not always meet the same
    // residue of the tile number modulo 8, i.e. the same address bits: how fast an XCD streams
    // depends on which part of memory it reads.
    constexpr int kRot = 37;
    const int bx = blockIdx.x;
    const int grid = phase1_participants(total_tiles, gridDim.x);  // g1
    auto slot_in_round = [&](int n) { return (bx + n * kRot) % grid; };
    const int full_rounds = grid > 0 ? total_tiles / grid : 0;
    const int n_mine = bx < grid ? full_rounds + (full_rounds * grid + slot_in_round(full_rounds) < total_tiles ? 1 : 0) : 0;
    auto tile_id = [&](int n) { return n * grid + slot_in_round(n); };

    const KSplit ks(H / 64, wave);  // ks.per <= kXSteps
    const int n_valid = ks.n_valid, kstride = ks.stride;
    const size_t k0 = n_valid > 0 ? ks.k0 : 0;  // a wavefront without steps re-reads the row's start
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    if (n_mine == 0) return;

    // Weight stream over this workgroup's tiles, P steps ahead, across expert boundaries; requests
    // past the last tile re-read it.
    u32x4 lo1[P], hi1[P], lo3[P], hi3[P];
    int is = 0, itile = 0;
    size_t wlo = 0, whi = 0;
    auto enter_tile = [&]() {
        const int id = tile_id(min(itile, n_mine - 1));
        const int d = id / tiles_per_expert;
        const size_t row0 = (size_t)g.expert[d] * F + (id - d * tiles_per_expert) * 16;
        wlo = (row0 + lm.row_lo) * H + k0 + lm.k_ld;
        whi = (row0 + lm.row_hi) * H + k0 + lm.k_ld;
    };
    enter_tile();
    auto issue = [&](int i) {
        const size_t off = (size_t)(is < n_valid ? is : 0) * kstride;
        lo1[i] = load16(p.w1 + wlo + off);
        hi1[i] = load16(p.w1 + whi + off);
        lo3[i] = load16(p.w3 + wlo + off);
        hi3[i] = load16(p.w3 + whi + off);
        if (++is == kXSteps) {
            is = 0;
            ++itile;
            enter_tile();
        }
    };
#pragma unroll
    for (int i = 0; i < P; ++i) issue(i);

    u32x4 xr[kXSteps][NC][2];  // token fragments of the current expert
    const int d_a = (g.n_active + 1) / 2;  // experts [0, d_a) of the active list are group A
    int cur_d = -1, par = 0;
    for (int ctile = 0; ctile < n_mine; ++ctile) {
        const int id = tile_id(ctile);
        const int d = id / tiles_per_expert;
        const int f0 = (id - d * tiles_per_expert) * 16;
        const int cnt = g.cnt[d];
        if (a_open && d >= d_a) {  // this workgroup's part of group A is complete
            announce(&p.flags[blockIdx.x], epoch);
            a_open = false;
        }
        if (d != cur_d) {
            cur_d = d;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                // columns without a token read the expert's first token (their results are unused)
                const uint16_t* xp = token_row<ALT, NC>(p, sm, g.assign[d][col + 16 * c < cnt ? col + 16 * c : 0]) + k0 + lm.kq8;
#pragma unroll
                for (int s = 0; s < kXSteps; ++s) {
                    const size_t off = (size_t)(s < n_valid ? s : 0) * kstride;
                    xr[s][c][0] = keep_if(s < n_valid, load16(xp + off));
                    xr[s][c][1] = keep_if(s < n_valid, load16(xp + off + 32));
                }
            }
        }
        f32x4 g1[NC], g2[NC], u1[NC], u2[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) g1[c] = g2[c] = u1[c] = u2[c] = zero;
#pragma unroll
        for (int s = 0; s < kXSteps; ++s) {
            const int i = s % P;
            bf16x8 a1, a2, a3, a4;
            mfma_operands(lm, lo1[i], hi1[i], a1, a2);
            mfma_operands(lm, lo3[i], hi3[i], a3, a4);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const bf16x8 b1 = __builtin_bit_cast(bf16x8, xr[s][c][0]);
                const bf16x8 b2 = __builtin_bit_cast(bf16x8, xr[s][c][1]);
                g1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1, g1[c], 0, 0, 0);
                g2[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, b2, g2[c], 0, 0, 0);
                u1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a3, b1, u1[c], 0, 0, 0);
                u2[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a4, b2, u2[c], 0, 0, 0);
            }
            issue(i);
        }
        // Tile done: fold the 8 K-slices.  MFMA 16x16 result: lane holds column (token)
        // lane & 15 and rows (features) 4 * (lane / 16) + r, r = 0..3.
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            sm.red[par][wave][0][c][lane] = fold_halves(g1[c], g2[c]);
            sm.red[par][wave][1][c][lane] = fold_halves(u1[c], u2[c]);
        }
        lds_barrier();
        for (int item = tid; item < 128 * NC; item += kThreads) {
            const int c = item >> 7, pl = item & 63, rp = (item >> 6) & 1;
            const int tok = (pl & 15) + 16 * c;
            if (tok < cnt) {
                float o[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float gs = 0.f, us = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        gs += sm.red[par][w][0][c][pl][2 * rp + h];
                        us += sm.red[par][w][1][c][pl][2 * rp + h];
                    }
                    o[h] = swiglu(gs, us);
                }
                // device-scope (write-through) store: read by other workgroups after the grid barrier
                uint32_t* dst = reinterpret_cast<uint32_t*>(p.act + (size_t)g.assign[d][tok] * F + f0 +
                                                            4 * (pl >> 4) + 2 * rp);
                __hip_atomic_store(dst, pack_bf16x2(o[0], o[1]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (Smem<NC>::kRedBufs == 1) lds_barrier();
        par = (par + 1) % Smem<NC>::kRedBufs;
    }
}

// ---- phase 2: y[t, h] = sum over the token's experts (ascending expert id) of
// w[a] * (act[a] . w2[e, h]) for this workgroup's 16-row tiles of h.  The first P steps of weight
// loads are issued before the grid-wide barrier that `act` has to wait for.
template <int P, int NC>
__device__ inline void gemm2_phase(const DecodeArgs& p, Smem<NC>& sm, uint32_t epoch, bool a_open) {
    const Groups<NC>& g = sm.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15;
    const LaneMap lm(lane);
    const int H = p.H, F = p.F, k = p.k;
    const int n_wgs = gridDim.x;

    const int h_tiles = H / 16;
    const int my_tiles = blockIdx.x < h_tiles ? (h_tiles - 1 - blockIdx.x) / n_wgs + 1 : 0;
    const KSplit ks(F / 64, wave);
    const int n_valid = ks.n_valid, kstride = ks.stride;
    const int spt = (ks.per + P - 1) / P * P;
    const int D = g.n_active;
    const long total_q = (long)my_tiles * D * spt;
    const size_t k0 = n_valid > 0 ? ks.k0 : 0;  // a wavefront without steps re-reads the row's start

    // ---- everything this workgroup stored to `act` has left the CU: raise flag B (and flag A, if
    // phase 1 did not get to it)
    const int d_a = (D + 1) / 2;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        if (a_open) __hip_atomic_store(&p.flags[blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&p.flags[kFlagStride + blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (total_q == 0) return;

    u32x4 lo[P], hi[P], aa[P][NC], ab[P][NC];
    // weight-side issue state
    int ws = 0, wd = 0, wt = blockIdx.x;
    size_t wlo = 0, whi = 0;
    auto enter_w = [&]() {
        const size_t row0 = (size_t)g.expert[wd] * H + wt * 16;
        wlo = (row0 + lm.row_lo) * F + k0 + lm.k_ld;
        whi = (row0 + lm.row_hi) * F + k0 + lm.k_ld;
    };
    enter_w();
    auto issue_w = [&](int i) {  // requests past the last tile re-read it
        const size_t off = (size_t)(ws < n_valid ? ws : 0) * kstride;
        lo[i] = load16(p.w2 + wlo + off);
        hi[i] = load16(p.w2 + whi + off);
        if (++ws == spt) {
            ws = 0;
            if (++wd == D) {
                wd = 0;
                wt += n_wgs;
            }
            if (wt < h_tiles) enter_w();
        }
    };
    // act-side issue state (the operand does not depend on the h tile)
    int as = 0, ad = 0;
    bool b_open = d_a < D;  // group B still has to be awaited
    size_t abase[NC];
    auto enter_a = [&]() {
#pragma unroll
        for (int c = 0; c < NC; ++c)  // columns without a token read the expert's first token (result unused)
            abase[c] = (size_t)g.assign[ad][col + 16 * c < g.cnt[ad] ? col + 16 * c : 0] * F + k0 + lm.kq8;
    };
    enter_a();
    auto issue_a = [&](int i) {
        const size_t off = (size_t)(as < n_valid ? as : 0) * kstride;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            aa[i][c] = load16(p.act + abase[c] + off);
            ab[i][c] = load16(p.act + abase[c] + off + 32);
        }
        if (++as == spt) {
            as = 0;
            if (++ad == D) ad = 0;
            if (b_open && ad >= d_a) {  // the next operand belongs to group B
                await_flags(p.flags + kFlagStride, n_wgs, epoch, p.spin_limit, p.flags + kStatusIndex, &sm.failed);
                b_open = false;
            }
            enter_a();
        }
    };
#pragma unroll
    for (int i = 0; i < P; ++i) issue_w(i);

    // ---- group A of the intermediate is needed now
    await_flags(p.flags, n_wgs, epoch, p.spin_limit, p.flags + kStatusIndex, &sm.failed);
#pragma unroll
    for (int i = 0; i < P; ++i) issue_a(i);

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 acc1[NC], acc2[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc1[c] = acc2[c] = zero;
    int cs = 0, cd = 0, ct = blockIdx.x, par = 0;
    for (long q = 0; q < total_q; q += P) {
#pragma unroll
        for (int i = 0; i < P; ++i) {
            bf16x8 a1, a2;
            mfma_operands(lm, lo[i], hi[i], a1, a2);
            const bool real = cs + i < n_valid;  // a padding step multiplies zeros
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                acc1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, __builtin_bit_cast(bf16x8, keep_if(real, aa[i][c])),
                                                                  acc1[c], 0, 0, 0);
                acc2[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8, keep_if(real, ab[i][c])),
                                                                  acc2[c], 0, 0, 0);
            }
            issue_w(i);
            issue_a(i);
        }
        cs += P;
        if (cs == spt) {
#pragma unroll
            for (int c = 0; c < NC; ++c) sm.red[par][wave][0][c][lane] = fold_halves(acc1[c], acc2[c]);
            lds_barrier();
            const int cnt = g.cnt[cd];
            for (int item = tid; item < 256 * NC; item += kThreads) {
                const int c = item >> 8, pl = item & 63, r = (item >> 6) & 3;
                const int tok = (pl & 15) + 16 * c;
                if (tok < cnt) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) s += sm.red[par][w][0][c][pl][r];
                    const int a = g.assign[cd][tok];
                    sm.yacc[a / k][4 * (pl >> 4) + r] += sm.w[a] * s;
                }
            }
            if (Smem<NC>::kRedBufs == 1) lds_barrier();  // the single buffer is free again
#pragma unroll
            for (int c = 0; c < NC; ++c) acc1[c] = acc2[c] = zero;
            cs = 0;
            par = (par + 1) % Smem<NC>::kRedBufs;
            if (++cd == D) {
                lds_barrier();  // the tile's sums are complete
                const bool failed = sm.failed != 0;
                for (int item = tid; item < p.T * 16; item += kThreads) {
                    const int t = item >> 4, r = item & 15;
                    p.y[(size_t)t * H + ct * 16 + r] = failed ? (uint16_t)0x7FC0 : to_bf16(sm.yacc[t][r]);
                    sm.yacc[t][r] = 0.f;
                }
                cd = 0;
                ct += n_wgs;
            }
        }
    }
}

// The whole MoE layer of a decode-size call in one launch (NC = 1, ROUTE), or the expert FFN of a
// call of up to 16 * NC tokens whose selections were made earlier.  Every workgroup must be
// resident at the same time (grid <= number of compute units, one 512-thread workgroup each).
template <int P1, int P2, bool ROUTE, int NC, bool ALT = false>
__global__ __launch_bounds__(kThreads) void decode_layer_kernel(DecodeArgs p) {
    static_assert(!ROUTE || NC == 1, "in-kernel routing serves at most 16 tokens");
    static_assert(!(ROUTE && ALT), "pre-calculated selections come with their routing");
    __shared__ Smem<NC> sm;
    const int tid = threadIdx.x;
    const int A = p.T * p.k;
    // The launch's epoch: read before anything of this launch can have changed the word.  What the
    // flags carry is the epoch mixed with a constant, so that leftovers of other uses of the memory
    // (small integers, zeros, all-ones) do not look like raised flags.
    // (Requested here, used after the routing, so its latency costs nothing.)
    const uint32_t last_count = __hip_atomic_load(&p.flags[kEpochIndex], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::: "memory");
    for (int i = tid; i < 16 * NC * 16; i += kThreads) sm.yacc[i >> 4][i & 15] = 0.f;
    if (tid == 0) sm.failed = 0;
    if (ROUTE) {
        // Every workgroup routes the call itself (identical arithmetic, identical result), which
        // costs a few microseconds of latency instead of a kernel boundary; workgroup 0 publishes.
        int old_count = 0;
        const bool publish = blockIdx.x == 0;
        if (publish && tid < p.E && p.accumulate) old_count = p.counts[tid];
        static_assert(sizeof(sm.red) >= kRoutePartFloats * sizeof(float), "routing borrows the reduction buffer");
        route_tokens_wg<uint16_t>(p.x, p.wg, p.bias, p.T, p.H, p.E, p.k, sm.route,
                                  reinterpret_cast<float*>(&sm.red[0][0][0][0][0]));
        if (tid < A) {
            sm.idx[tid] = sm.route.idx[tid];
            sm.w[tid] = sm.route.w[tid];
        }
        if (publish) {
            if (tid < A) {
                p.idx_out[tid] = sm.route.idx[tid];
                p.w_out[tid] = sm.route.w[tid];
            }
            if (tid < p.E) {
                int c = 0;
                for (int a = 0; a < A; ++a) c += sm.route.idx[a] == tid;
                p.counts[tid] = old_count + c;
            }
        }
    } else {
        for (int i = tid; i < A; i += kThreads) {
            sm.idx[i] = p.idx_in[i];
            sm.w[i] = p.w_in[i];
            if (ALT) sm.stale[i] = p.stale[i];
        }
    }
    __syncthreads();
    if (!ROUTE && p.counts != nullptr && blockIdx.x == 0 && tid < p.E) {
        // activation counts of selections made by a routing kernel before this one (17 to 32 tokens)
        int c = p.accumulate ? p.counts[tid] : 0;
        for (int a = 0; a < A; ++a) c += sm.idx[a] == tid;
        p.counts[tid] = c;
    }
    build_groups<NC>(sm.g, sm.idx, A, p.E);
    const uint32_t count = (uint32_t)__builtin_amdgcn_readfirstlane((int)last_count) + 1u;
    const uint32_t epoch = count ^ 0x9E3779B9u;
    bool a_open = true;  // flag A not raised yet
    if (p.H <= 64 * kXSteps * kWaves) gemm1_phase_xreg<P1, NC, ALT>(p, sm, epoch, a_open);
    else gemm1_phase<P1, NC, ALT>(p, sm, epoch, a_open);
    gemm2_phase<P2, NC>(p, sm, epoch, a_open);
    if (blockIdx.x == 0 && tid == 0)  // the next launch counts on from here
        __hip_atomic_store(&p.flags[kEpochIndex], count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ROUTE && p.wg_next != nullptr && blockIdx.x == gridDim.x - 1) {
        // The prediction for the next layer, which nothing in this call waits for: one workgroup
        // evaluates the next gate once its share of the experts is done (same routine as the routing
        // above, so the result is the one a separate routing call gives).
        __syncthreads();  // the reduction buffer is free
        route_tokens_wg<uint16_t>(p.x, p.wg_next, p.bias_next, p.T, p.H, p.E, p.k, sm.route,
                                  reinterpret_cast<float*>(&sm.red[0][0][0][0][0]));
        if (tid < A) p.pred_out[tid] = sm.route.idx[tid];
    }
}

}  // namespace

hipError_t launch_decode_layer(const moe_shape_t& s, int tokens, const void* x, const DecodeRoute* route,
                               const int32_t* topk_idx, const float* topk_w, const void* w1, const void* w3,
                               const void* w2, void* y, void* act, uint32_t* flags, const StaleInput& alt,
                               hipStream_t stream, int32_t* counts, int accumulate) {
    DecodeArgs p{};
    p.x_stale = static_cast<const uint16_t*>(alt.x_stale);
    p.stale = alt.stale;
    p.x = static_cast<const uint16_t*>(x);
    if (route != nullptr) {
        p.wg = static_cast<const uint16_t*>(route->w_gate);
        p.bias = route->bias;
        p.idx_out = route->idx;
        p.w_out = route->wts;
        p.counts = route->counts;
        p.accumulate = route->accumulate;
        p.wg_next = static_cast<const uint16_t*>(route->w_gate_next);
        p.bias_next = route->bias_next;
        p.pred_out = route->pred_idx;
    } else {
        p.idx_in = topk_idx;
        p.w_in = topk_w;
        p.counts = counts;
        p.accumulate = accumulate;
    }
    p.w1 = static_cast<const uint16_t*>(w1);
    p.w3 = static_cast<const uint16_t*>(w3);
    p.w2 = static_cast<const uint16_t*>(w2);
    p.act = static_cast<uint16_t*>(act);
    p.y = static_cast<uint16_t*>(y);
    p.flags = flags;
    p.spin_limit = decode_spin_limit();
    p.T = tokens;
    p.k = s.top_k;
    p.E = s.n_experts;
    p.H = s.hidden;
    p.F = s.ffn;
    const int max_tiles1 = min(s.n_experts, tokens * s.top_k) * (s.ffn / 16);
    const int grid = min(min(compute_units(), kFlagStride), max(max_tiles1, s.hidden / 16));
    if (route != nullptr) {
        decode_layer_kernel<kP1, kP2, true, 1><<<grid, kThreads, 0, stream>>>(p);
    } else if (alt.stale != nullptr) {
        if (tokens <= 16) decode_layer_kernel<kP1, kP2, false, 1, true><<<grid, kThreads, 0, stream>>>(p);
        else decode_layer_kernel<kP1, kP2, false, 2, true><<<grid, kThreads, 0, stream>>>(p);
    } else if (tokens <= 16) {
        decode_layer_kernel<kP1, kP2, false, 1><<<grid, kThreads, 0, stream>>>(p);
    } else {
        decode_layer_kernel<kP1, kP2, false, 2><<<grid, kThreads, 0, stream>>>(p);
    }
    stage_mark(stream, kStageFused);
    return hipGetLastError();
}

}  // namespace moe
