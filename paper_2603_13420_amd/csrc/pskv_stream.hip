// Streamed-prefix MFMA kernels of batched candidate-suffix attention for gfx950
// (bf16 tensors, head dim 128, prefix of any length).
//
// Used when the prefix K/V of one head does not fit in LDS.  The stacked query rows
//     r = (b*S + i)*G + g      (suffix-centric alignment, Sec. 4.3)
// of one KV head are cut into groups of 256; a "pass" is one (KV head, group) pair.  A
// persistent workgroup of 8 wavefronts takes passes in turn; each wavefront owns one 32-row
// block of the group and all eight walk over the prefix together, tile by tile: the 512 threads
// request the coming 32-key tiles of the single shared prefix K/V (Sec. 4.2: one copy for all
// candidates) from L2 straight into a small ring of fragment-major LDS images while the current
// tiles are being used, and meet at one barrier per two tiles.  Every tile is thus
// read once per 256 rows, whatever candidates those rows belong to, and the prefix itself is
// read from HBM about once per XCD: pass ids are laid out so that the workgroups of one XCD
// (workgroup ids go round the XCDs) work on one head at a time, and find it in that XCD's L2.
//
// Three kernels.  The pipelined one (every 32-row block inside one candidate) is the software
// pipeline of the resident-prefix kernel with the tile images taken from the ring, the suffix
// handled after the prefix, and a fixed per-row reference maximum; when a row turns out to
// need rescaling, the workgroup repeats its passes on the general path.  The general one
// (any shape) is the classic online softmax, one tile at a time.  The third (further down) is
// for suffix-side segments of several tiles: its passes are cut out of one candidate, whose own
// suffix K/V then goes through the ring like the prefix.
// Operand layouts and the pieces shared with the resident kernels are in pskv_mfma.hpp.
#include "pskv_mfma.hpp"

namespace pskv {
namespace {

constexpr int kRing = 8;                   // tile slots in LDS
constexpr int kSlotBytes = 2 * kTileBytes; // K image, then V image
constexpr int kLdsBytes = kRing * kSlotBytes + kNW * kScrBytes;
constexpr int kPassRows = kNW * kBlockRows;
constexpr int kMinTiles = 3;                // shortest prefix, in tiles, that the pipelined pass takes

typedef __attribute__((address_space(3))) int lds_int;

__device__ inline Ctx make_stream_ctx(const Args &a, lds_u8 *smem, int tid)
{
    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.Mtot = a.C * a.S * a.G;
    X.c = a.scale * kLog2e;
    X.k_lane = smem + X.lane * 16;             // slot 0; slot s is kSlotBytes*s further
    X.v_lane = smem + kTileBytes + X.lane * 8;
    X.scr = smem + kRing * kSlotBytes + __builtin_amdgcn_readfirstlane(tid >> 6) * kScrBytes;
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    set_vhead(a, X, 0);
    return X;
}

// ------------------------------------------------------------------------------------------
// General pass: classic online softmax, tiles double-buffered in slots 0 and 1.  Every thread
// of the workgroup must call it (barriers inside), whether or not its wavefront has a block.
// ------------------------------------------------------------------------------------------
__device__ __attribute__((always_inline)) void general_pass(const Args &a, Ctx &X, lds_u8 *smem, int tid, int vh, int blk,
                                                            bool active)
{
    set_vhead(a, X, vh);
    const int ntiles = (X.P + kTileKeys - 1) / kTileKeys;
    const TileSlot t = make_tile_slot(tid);
    const int r0 = blk * kBlockRows;
    const Row row = decode_row(a, X, blk);
    const bool rvalid = active && row.rin && (int)row.ri < clamp_len(a, row.rlen);
    const bool work = __builtin_amdgcn_ballot_w64(rvalid) != 0;
    uintx4 q[8];
    load_q(a, X, row, q);

    RowState st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            st.o[dt][e] = 0.f;

    if (ntiles > 0) {
        uintx4 kv, vv;
        load_tile_chunks(a, X, t, 0, kv, vv);
        __syncthreads(); // whatever the ring held has been used by every wavefront
        write_tile_chunks(X, t, 0, smem, smem + kTileBytes, tid, kv, vv);
        __syncthreads();
        for (int kt = 0; kt < ntiles; ++kt) {
            const int ktn = kt + 1 < ntiles ? kt + 1 : kt;
            load_tile_chunks(a, X, t, ktn, kv, vv);
            if (work)
                prefix_tile_classic(X, X.k_lane + (kt & 1) * kSlotBytes, X.v_lane + (kt & 1) * kSlotBytes,
                                    X.P - kt * kTileKeys, q, st);
            if (kt + 1 < ntiles) {
                lds_u8 *slot = smem + ((kt + 1) & 1) * kSlotBytes;
                write_tile_chunks(X, t, kt + 1, slot, slot + kTileBytes, tid, kv, vv);
            }
            __syncthreads();
        }
    }
    if (active) {
        if (work) {
            suffix_classic(a, X, r0, row, q, st);
            store_block(a, X, r0, row, rvalid, st.m, st.l, st.o);
        } else {
            store_zero_block(a, X, r0, row);
        }
    }
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void stream_general_kernel(Args a, int npasses)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    Ctx X = make_stream_ctx(a, smem, tid);
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    for (int p = blockIdx.x; p < npasses; p += gridDim.x) {
        const Pass ps = make_pass(a, p, npasses, nblocks, wave);
        if (ps.exists)
            general_pass(a, X, smem, tid, ps.vh, ps.blk, ps.active);
    }
}

// ------------------------------------------------------------------------------------------
// Pipelined passes.  Preconditions (checked by the launcher): S*G is a multiple of 32, so a
// 32-row block lies inside one candidate; the padded prefix has at least three tiles; one head's prefix
// spans less than 2^31 bytes, so tile addresses are a scalar base plus a 32-bit lane offset.
// ONE_STEP: S <= 32, the suffix is a single 32-key step.
//
// Ring protocol.  Step t of a pass (see pipe_tile) reads the K images of tiles t+1 and t+2 and
// the V images of tiles t-1 and t.  Steps are taken two at a time.  Tiles are requested with
// direct-to-LDS loads, tile u into slot u % 8, tiles 0..6 at the start of the pass.  At the top
// of the pair (t, t+1) every thread waits until its requests for the tiles up to t+3 have landed
// (the vector memory counter retires requests in order: all but those of tile t+4 must be
// complete), the workgroup meets at a barrier - after which everybody's parts of those tiles are
// there and nobody reads tiles up to t-2 any more - and tiles t+5 and t+6 are requested into the
// slots of tiles t-3 and t-2.  The pair then reads tiles t-1 .. t+3.
// Rows past the end of a ragged last tile are fetched from the last prefix row instead: their
// scores are masked and their weights are exactly zero, so finite data is all that is needed.
// ------------------------------------------------------------------------------------------
struct Stager {
    const unsigned char *kbase, *vbase; // this head's prefix K and V (wave-uniform)
    unsigned k_off, v_off;              // this thread's chunk within a full tile, bytes
    unsigned k_off_last, v_off_last;    // ... within the last tile (rows clamped into the prefix)
    unsigned tile_stride;               // bytes from one tile to the next
    int last;                           // index of the last tile
};

// One 16-byte request per lane straight into LDS: lane l's bytes, fetched from gbase + voff (gbase
// the same for the whole wavefront and held in scalar registers, voff the lane's own 32-bit
// offset), land at lds_base + 16*l (lds_base is the same for the whole wavefront).
// Written as an instruction rather than through the
// compiler's builtin: the compiler would make every later LDS read wait for all such requests
// still in flight.  Its own bookkeeping of the vector memory counter stays on the safe side:
// requests it does not know of can only make its waits longer.  M0 carries the LDS address and
// is declared clobbered: the statement then counts as a write of M0 for the compiler's passes
// that merge and hoist its own M0 set-ups, which keeps them from moving one across it.  (M0 is a
// reserved register, never allocated, which is all the warning silenced here has to say.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void request_to_lds(const unsigned char *gbase, unsigned voff, lds_u8 *lds_base)
{
    const unsigned lds_addr = (unsigned)(unsigned long long)lds_base;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
// s_waitcnt immediate (gfx9 encoding): vector memory counter at most n (n < 16), the others untouched
#define PSKV_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | (n))

template <bool ONE_STEP>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void stream_pipelined_kernel(Args a, int npasses)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    Ctx X = make_stream_ctx(a, smem, tid);
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    auto kimg = [&](int t) { return X.k_lane + (t & (kRing - 1)) * kSlotBytes; };
    auto vimg = [&](int t) { return X.v_lane + (t & (kRing - 1)) * kSlotBytes; };
    // this thread's two requests for tile kt (kt <= the last tile), straight into slot kt % 8
    auto request = [&](const Stager &g, int kt) {
        const unsigned base = (unsigned)kt * g.tile_stride;
        lds_u8 *slot = smem + (kt & (kRing - 1)) * kSlotBytes + wave * 1024;
        request_to_lds(g.kbase + base, kt == g.last ? g.k_off_last : g.k_off, slot);
        request_to_lds(g.vbase + base, kt == g.last ? g.v_off_last : g.v_off, slot + kTileBytes);
    };

    Stager g;
    const TileSlot ts = make_tile_slot(tid);
    g.k_off = (unsigned)(ts.k_row * a.kp_sp + ts.k_chunk * 8) * 2u;
    g.v_off = (unsigned)(ts.v_row * a.kp_sp + ts.v_chunk * 8) * 2u;
    g.tile_stride = (unsigned)(kTileKeys * a.kp_sp) * 2u;

    bool wg_bad = false;
    int p = blockIdx.x;
    Pass ps = make_pass(a, p, npasses, nblocks, wave);
    BlockRows nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
    uintx4 q[8]; // this pass's Q fragments until their last use, then the next pass's
    load_q_block(a, X, nxt, q);

    bool wg_short = false;
    while (p < npasses) {
        set_vhead(a, X, ps.vh);
        const int T = (X.P + kTileKeys - 1) / kTileKeys;
        if (!ps.exists || T < kMinTiles) { // nothing here, or this instruction's prefix is too short for the pipeline:
                                           // left to the general sweep below
            wg_short |= ps.exists;
            p += gridDim.x;
            ps = make_pass(a, p, npasses, nblocks, wave);
            nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
            load_q_block(a, X, nxt, q);
            continue;
        }
        {
            const int nlast = X.P - (T - 1) * kTileKeys; // rows of the last tile, 1..32
            const int kr = ts.k_row < nlast ? ts.k_row : nlast - 1, vr = ts.v_row < nlast ? ts.v_row : nlast - 1;
            g.k_off_last = (unsigned)(kr * a.kp_sp + ts.k_chunk * 8) * 2u;
            g.v_off_last = (unsigned)(vr * a.kp_sp + ts.v_chunk * 8) * 2u;
            g.last = T - 1;
            g.kbase = reinterpret_cast<const unsigned char *>(X.kpg);
            g.vbase = reinterpret_cast<const unsigned char *>(X.vpg);
        }
        const int blk = ps.blk, r0 = blk * kBlockRows;
        const bool active = ps.active;
        const BlockRows row = nxt;
        const bool rvalid = active && row.ri < row.len;

        // The ring is free here: the barrier that ended the previous pass was passed only by
        // wavefronts that had finished reading it.  Tiles 0..6 are requested at once; the first
        // steps need tiles 0..3.
#pragma unroll
        for (int u = 0; u < 7; ++u)
            if (u < T)
                request(g, u);
        if (T >= 7)
            PSKV_WAIT_VM(6);
        else
            PSKV_WAIT_VM(0);
        __syncthreads();
        // Top of the pair (t, t+1): tiles up to t+3 have landed for everyone (tile t+4 may still be
        // in flight); nobody reads tiles up to t-2 any more: their slots take tiles t+5 and t+6.
        auto pair_top = [&](int t) {
            if (t + 4 <= T - 1)
                PSKV_WAIT_VM(2);
            else
                PSKV_WAIT_VM(0);
            __syncthreads();
            if (t + 5 <= T - 1)
                request(g, t + 5);
            if (t + 6 <= T - 1)
                request(g, t + 6);
        };

        // the block's suffix: candidate sb, keys 0..skmax
        const int i_hi = (int)fdiv(r0 + kBlockRows - 1, a.div_g) - (row.b - X.cand0) * a.S;
        const int skmax = i_hi < row.len - 1 ? i_hi : row.len - 1;
        const int skld = skmax > 0 ? skmax : 0; // row the suffix loads are clamped to (a candidate may be empty)

        // ---- first prefix tile: scores, reference maximum ----
        floatx16 sA, sB; // raw scores of the current and of the next tile, roles alternating
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sA[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(kimg(0) + ks * 1024)), as_bf16x8(q[ks]), sA,
                                                         0, 0, 0);
        Pre pre;
#pragma unroll
        for (int i = 0; i < kDist; ++i)
            pre.k[i] = *(lds_u128 *)(kimg(1) + i * 1024);
        float m = sA[0];
#pragma unroll
        for (int e = 1; e < 16; ++e)
            m = fmaxf(m, sA[e]);
        m = fmaxf(m, __shfl_xor(m, 32, 64)) * X.c; // the other half-wave holds the other 16 keys
        float l = 0.f;
        floatx16 o[4];
        uintx4 pA[2], pB[2]; // packed weights of the current and of the previous tile, roles alternating
        uintx4 skf[8], svf[2][4];

        // ---- pipeline over the prefix tiles: step t = scores of tile t+1, weights of tile t,
        //      value product of tile t-1 ----
        pipe_tile<true, false, false, false, false, true, true>(kimg(1), skf, vimg(0), kimg(2), vimg(0), pre, q, sA, sB,
                                                                X.c, m, 0, l, pA, pA, o);
        pipe_tile<true, false, true, true, false, true, true>(kimg(2), skf, vimg(0), kimg(3), vimg(1), pre, q, sB, sA, X.c,
                                                              m, 0, l, pA, pB, o);
        // one pair of steps
#define PSKV_STEP_PAIR(t)                                                                                              \
    do {                                                                                                               \
        pipe_tile<true, false, true, false, false, true, true>(kimg((t) + 1), skf, vimg((t) - 1), kimg((t) + 2),       \
                                                               vimg(t), pre, q, sA, sB, X.c, m, 0, l, pB, pA, o);      \
        pipe_tile<true, false, true, false, false, true, true>(kimg((t) + 2), skf, vimg(t),                            \
                                                               kimg((t) + 3 < T ? (t) + 3 : T - 1), vimg((t) + 1),     \
                                                               pre, q, sB, sA, X.c, m, 0, l, pA, pB, o);               \
    } while (0)
        int t = 2;
        for (; t + 3 <= T - 2; t += 2) {
            pair_top(t);
            PSKV_STEP_PAIR(t);
        }
        // The last pair requests no further tiles; the suffix K fragments, needed two or three
        // steps from here, are requested once the staging registers are free.
        if (t + 1 <= T - 2) {
            pair_top(t);
            load_suffix_k_block(a, X, row.b, 0, skld, skf);
            PSKV_STEP_PAIR(t);
            t += 2;
        } else {
            load_suffix_k_block(a, X, row.b, 0, skld, skf);
        }
#undef PSKV_STEP_PAIR
        if (t <= T - 2) { // one step left over: do it and put scores and weights back in their places
            pipe_tile<true, false, true, false, false, true, true>(kimg(t + 1), skf, vimg(t - 1), kimg(T - 1), vimg(t), pre,
                                                                   q, sA, sB, X.c, m, 0, l, pB, pA, o);
            sA = sB;
            pB[0] = pA[0];
            pB[1] = pA[1];
        }
        if (X.P & (kTileKeys - 1)) { // ragged last prefix tile: keys past the prefix are not visible
            const int nv = X.P - (T - 1) * kTileKeys - 4 * X.h;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (8 * (e >> 2) + (e & 3) >= nv)
                    sA[e] = -INFINITY;
        }
        load_suffix_v_block(a, X, row.b, 0, skld, svf); // one step ahead of its use
        // ---- last prefix tile: the "next scores" are those of the first suffix step ----
        pipe_tile<true, true, true, false, false, false, true>(kimg(0), skf, vimg(T - 2), kimg(0), vimg(T - 1), pre, q, sA,
                                                               sB, X.c, m, 0, l, pB, pA, o);

        // the next pass of this workgroup (clamped past the end: requested unconditionally)
        p += gridDim.x;
        ps = make_pass(a, p, npasses, nblocks, wave);
        // Without further suffix steps (always so when S <= 32) Q has been used for the last time:
        // the next pass's Q takes its place.
        const bool more = !ONE_STEP && skmax >= kTileKeys;
        if (!more) {
            nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
            load_q_block(a, X, nxt, q);
        }

        // ---- first suffix step: causal mask and weights under the value product of the last
        //      prefix tile; then its own value product through the scratch tile ----
        pipe_tile<false, false, true, false, true, false, false>(kimg(0), skf, vimg(T - 1), kimg(0), vimg(0), pre, q, sB, sB,
                                                                 X.c, m, row.ri - 4 * X.h, l, pA, pB, o);
        pv_from_scratch(X, svf[0], as_bf16x8(pB[0]), o);
        pv_from_scratch(X, svf[1], as_bf16x8(pB[1]), o);
        if (more) {
            // The second suffix step's K and V and, in the same round trip to memory, the next
            // pass's Q (into registers of its own: this pass's Q is still needed for the scores).
            uintx4 qn[8];
            load_suffix_k_block(a, X, row.b, kTileKeys, skmax, skf);
            load_suffix_v_block(a, X, row.b, kTileKeys, skmax, svf);
            nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
            load_q_block(a, X, nxt, qn);
            for (int k0 = kTileKeys;; k0 += kTileKeys) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    sB[e] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(skf[ks]), as_bf16x8(q[ks]), sB, 0, 0, 0);
                const bool again = k0 + kTileKeys <= skmax;
                if (again)
                    load_suffix_k_block(a, X, row.b, k0 + kTileKeys, skmax, skf);
                suffix_step_fixed(X, row.ri, k0, sB, m, l, svf, o);
                if (!again)
                    break;
                load_suffix_v_block(a, X, row.b, k0 + kTileKeys, skmax, svf);
            }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                q[ks] = qn[ks];
        }

        const bool bad = __builtin_amdgcn_ballot_w64(rvalid && !(l < kBig)) != 0;
        if (active)
            store_block_rows(a, X, row, m, l, o);
        // the wavefront's verdict goes into the first word of its own scratch tile
        if (X.lane == 0)
            *(lds_int *)X.scr = bad ? 1 : 0;
        __syncthreads(); // ends the pass: the ring is free, the verdicts are visible
        wg_bad |= __builtin_amdgcn_ballot_w64(*(lds_int *)(smem + kRing * kSlotBytes + (X.lane & (kNW - 1)) * kScrBytes) !=
                                              0) != 0;
    }

    // Rare: some row met scores far above its first tile's maximum; whatever this workgroup
    // stored is then replaced by the general path's result.  The same sweep serves the passes
    // skipped above.  (Kept out of the main loop so that it costs it no registers.)
    if (wg_bad || wg_short)
        for (int p2 = blockIdx.x; p2 < npasses; p2 += gridDim.x) {
            const Pass ps2 = make_pass(a, p2, npasses, nblocks, wave);
            set_vhead(a, X, ps2.vh);
            if (ps2.exists && (wg_bad || (X.P + kTileKeys - 1) / kTileKeys < kMinTiles))
                general_pass(a, X, smem, tid, ps2.vh, ps2.blk, ps2.active);
        }
}

// ------------------------------------------------------------------------------------------
// Candidate passes: suffix-side segments of several 32-key tiles (suffix, template tail and
// target together, Sec. 3.1).  Here the causal part is no longer a small correction after the
// prefix, and fetching a candidate's suffix K/V per wavefront, one exposed round trip per tile,
// dominates.  So a pass is cut out of ONE candidate: (candidate, KV head, group of up to 8 of the
// candidate's S*G/32 row blocks), and the ring simply goes on after the last prefix tile with
// the 32-key tiles of that candidate's own suffix K/V, up to the last key any row of the pass
// sees.  Every tile, prefix or suffix, is then staged once per pass by all 512 threads, several
// tiles ahead of its use, and every step is a step of the same three-stage pipeline; a step
// whose tile has keys some row does not see (ragged last prefix tile, suffix tiles at or past
// the row's own position) takes the masked form of the step, the limit being per row.
// A tile wholly in a row's future gives that row weights of exactly zero.
//
// Pass ids are laid out so that the groups of one (candidate, KV head) unit run at the same
// time on compute units of one XCD (workgroup ids go round the XCDs): the unit's suffix K/V is
// then fetched from HBM once and found in that XCD's L2 by the other groups.
// Preconditions (launcher): those of the pipelined passes above, and S*ks_stride_s*2 < 2^31.
// ------------------------------------------------------------------------------------------
struct CandShape {
    int nblk_c; // 32-row blocks per candidate (S*G/32)
    int ngrp;   // passes per (candidate, KV head) unit
    int bpp;    // blocks per pass (the last pass of a unit may hold fewer)
};

struct CandPass {
    int vh, head, cand0; // as in Pass
    int b;               // candidate (global index)
    int cblk0, cblk_last; // first and last block of the pass within the candidate
    int blk;             // this wavefront's block in the instruction's row space (clamped)
    bool exists;         // the unit exists (unit ids are padded to a multiple of 8)
    bool active;         // the wavefront has a block
};

__device__ inline CandPass make_cand_pass(const Args &a, const CandShape &cs, int p, int npasses, int wave)
{
    CandPass ps;
    const int pc = p < npasses ? p : npasses - 1;
    const int q = pc >> 3, x = pc & 7;
    const int uq = q / cs.ngrp, grp = q - uq * cs.ngrp;
    const int units = a.B * a.Hkv;
    int u = uq * 8 + x;
    ps.exists = p < npasses && u < units;
    u = u < units ? u : units - 1;
    ps.b = u / a.Hkv;
    ps.head = u - ps.b * a.Hkv;
    const int n = ps.b / a.C;
    ps.vh = n * a.Hkv + ps.head;
    ps.cand0 = n * a.C;
    ps.cblk0 = grp * cs.bpp;
    const int rest = cs.nblk_c - ps.cblk0;
    const int nb = rest < cs.bpp ? rest : cs.bpp;
    ps.cblk_last = ps.cblk0 + nb - 1;
    ps.active = ps.exists && wave < nb;
    const int cblk = ps.cblk0 + wave;
    ps.blk = (ps.b - ps.cand0) * cs.nblk_c + (cblk < ps.cblk_last ? cblk : ps.cblk_last);
    return ps;
}

struct CandStager {
    const unsigned char *kp, *vp;       // prefix K and V of the pass's instruction and head
    const unsigned char *ks, *vs;       // suffix K and V of the pass's candidate and head
    unsigned k_off, v_off;              // prefix: this thread's chunk within a full tile, bytes
    unsigned k_off_last, v_off_last;    // ... within the last prefix tile (rows clamped into the prefix)
    unsigned tile_stride;               // bytes from one prefix tile to the next
    int k_row, v_row;                   // suffix: this thread's rows within a tile ...
    unsigned k_col, v_col, row_stride;  // ... byte offsets of its chunks within a row, bytes per row
    int Tp;                             // prefix tiles
    int last;                           // index of the pass's last tile, prefix and suffix tiles counted together
    int skmax;                          // last suffix key any row of the pass sees
};

// Tile kt of the pass (clamped to its last tile).  Suffix rows past skmax are fetched from row
// skmax: no valid row sees them, finite data is all that is needed.
__device__ inline void cand_stage_load(const CandStager &g, int kt, uintx4 &kv, uintx4 &vv)
{
    const int u = kt < g.last ? kt : g.last;
    if (u < g.Tp) {
        const unsigned base = (unsigned)u * g.tile_stride;
        const bool lastp = u == g.Tp - 1;
        kv = *reinterpret_cast<const uintx4 *>(g.kp + (base + (lastp ? g.k_off_last : g.k_off)));
        vv = *reinterpret_cast<const uintx4 *>(g.vp + (base + (lastp ? g.v_off_last : g.v_off)));
    } else {
        const int j0 = (u - g.Tp) * kTileKeys;
        const int kr = j0 + g.k_row < g.skmax ? j0 + g.k_row : g.skmax;
        const int vr = j0 + g.v_row < g.skmax ? j0 + g.v_row : g.skmax;
        kv = *reinterpret_cast<const uintx4 *>(g.ks + ((unsigned)kr * g.row_stride + g.k_col));
        vv = *reinterpret_cast<const uintx4 *>(g.vs + ((unsigned)vr * g.row_stride + g.v_col));
    }
}

// O^T += V^T P^T for one tile whose V image is in the ring.
__device__ inline void pv_tile(lds_u8 *v_img, const uintx4 (&pp)[2], floatx16 (&o)[4])
{
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        o[ks & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_fragment(v_img, ks & 3, ks >> 2), as_bf16x8(pp[ks >> 2]),
                                                            o[ks & 3], 0, 0, 0);
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void stream_candidate_kernel(Args a, int npasses, CandShape cs)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    Ctx X = make_stream_ctx(a, smem, tid);
    auto kimg = [&](int t) { return X.k_lane + (t & (kRing - 1)) * kSlotBytes; };
    auto vimg = [&](int t) { return X.v_lane + (t & (kRing - 1)) * kSlotBytes; };
    auto stage_write = [&](int kt, const uintx4 &kv, const uintx4 &vv) {
        lds_u8 *slot = smem + (kt & (kRing - 1)) * kSlotBytes + tid * 16;
        *(lds_u128 *)slot = kv;
        *(lds_u128 *)(slot + kTileBytes) = vv;
    };

    CandStager g;
    const TileSlot ts = make_tile_slot(tid);
    g.k_off = (unsigned)(ts.k_row * a.kp_sp + ts.k_chunk * 8) * 2u;
    g.v_off = (unsigned)(ts.v_row * a.kp_sp + ts.v_chunk * 8) * 2u;
    g.tile_stride = (unsigned)(kTileKeys * a.kp_sp) * 2u;
    g.k_row = ts.k_row;
    g.v_row = ts.v_row;
    g.k_col = (unsigned)ts.k_chunk * 16u;
    g.v_col = (unsigned)ts.v_chunk * 16u;
    g.row_stride = (unsigned)a.ks_ss * 2u;

    bool wg_bad = false, wg_short = false;
    int p = blockIdx.x;
    CandPass ps = make_cand_pass(a, cs, p, npasses, wave);
    BlockRows nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
    uintx4 q[8]; // this pass's Q fragments until their last use, then the next pass's
    load_q_block(a, X, nxt, q);

    while (p < npasses) {
        set_vhead(a, X, ps.vh);
        const int Tp = (X.P + kTileKeys - 1) / kTileKeys;
        const int len = len_uniform(a, ps.b);
        const int i_lo = (int)fdiv(ps.cblk0 * kBlockRows, a.div_g); // first suffix position of the pass
        const bool nothing = !ps.exists || i_lo >= len;             // no unit, or nothing but padding
        if (nothing || Tp < kMinTiles) {
            if (!nothing)
                wg_short = true; // prefix too short for the pipeline: left to the general sweep below
            else if (ps.active)
                store_zero_block_rows(a, X, nxt);
            p += gridDim.x;
            ps = make_cand_pass(a, cs, p, npasses, wave);
            nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
            load_q_block(a, X, nxt, q);
            continue;
        }
        const int i_hi = (int)fdiv(ps.cblk_last * kBlockRows + kBlockRows - 1, a.div_g);
        const int skmax = i_hi < len - 1 ? i_hi : len - 1;
        const int T = Tp + skmax / kTileKeys + 1;
        {
            const int nlast = X.P - (Tp - 1) * kTileKeys; // rows of the last prefix tile, 1..32
            const int kr = ts.k_row < nlast ? ts.k_row : nlast - 1, vr = ts.v_row < nlast ? ts.v_row : nlast - 1;
            g.k_off_last = (unsigned)(kr * a.kp_sp + ts.k_chunk * 8) * 2u;
            g.v_off_last = (unsigned)(vr * a.kp_sp + ts.v_chunk * 8) * 2u;
            g.Tp = Tp;
            g.last = T - 1;
            g.skmax = skmax;
            g.kp = reinterpret_cast<const unsigned char *>(X.kpg);
            g.vp = reinterpret_cast<const unsigned char *>(X.vpg);
            g.ks = reinterpret_cast<const unsigned char *>(X.ksg + (long long)ps.b * a.ks_sb);
            g.vs = reinterpret_cast<const unsigned char *>(X.vsg + (long long)ps.b * a.ks_sb);
        }
        const BlockRows row = nxt;
        // This wavefront's own share of the pass's tiles: the prefix and the suffix tiles up to the
        // last key its own block sees (Tw <= T); none at all if it has no block or its block holds
        // nothing but padding (then it only stores zeros).
        const int cblk = ps.blk - (ps.b - ps.cand0) * cs.nblk_c; // block within the candidate
        const int i_lo_w = (int)fdiv(cblk * kBlockRows, a.div_g);
        const int i_hi_w = (int)fdiv(cblk * kBlockRows + kBlockRows - 1, a.div_g);
        const bool active = ps.active && i_lo_w < len;
        const int Tw = Tp + (i_hi_w < skmax ? i_hi_w : skmax) / kTileKeys + 1;
        const bool rvalid = active && row.ri < row.len;

        // The ring is free here (the barrier that ended the previous pass).  Tiles 0..3 go in at once.
        uintx4 kv0, vv0, kv1, vv1;
        {
            uintx4 kv2, vv2, kv3, vv3;
            cand_stage_load(g, 0, kv0, vv0);
            cand_stage_load(g, 1, kv1, vv1);
            cand_stage_load(g, 2, kv2, vv2);
            cand_stage_load(g, 3, kv3, vv3);
            stage_write(0, kv0, vv0);
            stage_write(1, kv1, vv1);
            stage_write(2, kv2, vv2);
            stage_write(3, kv3, vv3);
        }
        cand_stage_load(g, 4, kv0, vv0);
        cand_stage_load(g, 5, kv1, vv1);
        __syncthreads();

        // Visibility limit of tile t for this lane's row, as pipe_tile takes it: element e (key
        // offset 8*(e/4) + e%4 + 4*h within the tile) is visible iff its offset without the
        // 4*h is <= lim.  Prefix tiles are fully visible but for the end of a ragged last one;
        // suffix tile j holds keys 32*j.. of which the row sees those up to its own position.
        const int lim_suffix = row.ri - 4 * X.h + Tp * kTileKeys;
        const int lim_last_prefix = X.P - (Tp - 1) * kTileKeys - 1 - 4 * X.h;
        auto lim_of = [&](int t) { return t >= Tp ? lim_suffix - t * kTileKeys : (t == Tp - 1 ? lim_last_prefix : 1 << 20); };
        const int tm = X.P / kTileKeys; // first tile with keys that some row does not see (>= 2)

        // A wavefront without a block (the last pass of a unit may hold fewer than eight) takes part
        // in the staging and in the barriers only, and leaves the matrix cores of its SIMD to its
        // neighbour: same barriers, in the same order, as the path below.
        if (!active) {
            if (ps.active)
                store_zero_block_rows(a, X, row);
            for (int t = 2; t + 1 <= T - 2; t += 2) {
                stage_write(t + 2, kv0, vv0);
                stage_write(t + 3, kv1, vv1);
                cand_stage_load(g, t + 4, kv0, vv0);
                cand_stage_load(g, t + 5, kv1, vv1);
                __syncthreads();
            }
            p += gridDim.x;
            ps = make_cand_pass(a, cs, p, npasses, wave);
            nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
            load_q_block(a, X, nxt, q);
            if (X.lane == 0)
                *(lds_int *)X.scr = 0;
            __syncthreads(); // ends the pass
            wg_bad |= __builtin_amdgcn_ballot_w64(*(lds_int *)(smem + kRing * kSlotBytes + (X.lane & (kNW - 1)) * kScrBytes) !=
                                                  0) != 0;
            continue;
        }

        // ---- first prefix tile: scores, reference maximum ----
        floatx16 sA, sB;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sA[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(kimg(0) + ks * 1024)), as_bf16x8(q[ks]), sA,
                                                         0, 0, 0);
        Pre pre;
#pragma unroll
        for (int i = 0; i < kDist; ++i)
            pre.k[i] = *(lds_u128 *)(kimg(1) + i * 1024);
        float m = sA[0];
#pragma unroll
        for (int e = 1; e < 16; ++e)
            m = fmaxf(m, sA[e]);
        m = fmaxf(m, __shfl_xor(m, 32, 64)) * X.c;
        float l = 0.f;
        floatx16 o[4];
        uintx4 pA[2], pB[2];
        uintx4 nokf[8]; // stands in for the register K fragments no step here uses

        pipe_tile<true, false, false, false, false, true, true>(kimg(1), nokf, vimg(0), kimg(2), vimg(0), pre, q, sA, sB,
                                                                X.c, m, 0, l, pA, pA, o);
        pipe_tile<true, false, true, true, false, true, true>(kimg(2), nokf, vimg(0), kimg(3 < Tw ? 3 : Tw - 1), vimg(1), pre, q,
                                                              sB, sA, X.c, m, 0, l, pA, pB, o);
#define PSKV_CAND_PAIR(t, MASKED)                                                                                      \
    do {                                                                                                               \
        pipe_tile<true, false, true, false, MASKED, true, true>(kimg((t) + 1), nokf, vimg((t) - 1), kimg((t) + 2),     \
                                                                vimg(t), pre, q, sA, sB, X.c, m, lim_of(t), l, pB, pA, \
                                                                o);                                                    \
        pipe_tile<true, false, true, false, MASKED, true, true>(kimg((t) + 2), nokf, vimg(t),                          \
                                                                kimg((t) + 3 < Tw ? (t) + 3 : Tw - 1), vimg((t) + 1),  \
                                                                pre, q, sB, sA, X.c, m, lim_of((t) + 1), l, pA, pB,    \
                                                                o);                                                    \
    } while (0)
        int t = 2;
        for (; t + 1 <= Tw - 2 && t + 1 < tm; t += 2) { // pairs of fully visible tiles
            stage_write(t + 2, kv0, vv0);
            stage_write(t + 3, kv1, vv1);
            cand_stage_load(g, t + 4, kv0, vv0);
            cand_stage_load(g, t + 5, kv1, vv1);
            __syncthreads();
            PSKV_CAND_PAIR(t, false);
        }
        for (; t + 1 <= Tw - 2; t += 2) {
            stage_write(t + 2, kv0, vv0);
            stage_write(t + 3, kv1, vv1);
            cand_stage_load(g, t + 4, kv0, vv0);
            cand_stage_load(g, t + 5, kv1, vv1);
            __syncthreads();
            PSKV_CAND_PAIR(t, true);
        }
        const int t_own = t; // the wavefront's own tiles end here; staging for the others goes on below
#undef PSKV_CAND_PAIR
        if (t <= Tw - 2) { // one step left over: do it and put scores and weights back in their places
            pipe_tile<true, false, true, false, true, false, true>(kimg(t + 1), nokf, vimg(t - 1), kimg(Tw - 1), vimg(t), pre,
                                                                   q, sA, sB, X.c, m, lim_of(t), l, pB, pA, o);
            sA = sB;
            pB[0] = pA[0];
            pB[1] = pA[1];
        }

        // Q has been used for the last time: the next pass's Q takes its place
        p += gridDim.x;
        ps = make_cand_pass(a, cs, p, npasses, wave);
        nxt = decode_block(a, X, ps.blk, ps.head, ps.cand0);
        load_q_block(a, X, nxt, q);

        // ---- last tile: its weights under the value product of the tile before, then its own ----
        pipe_tile<false, false, true, false, true, false, false>(kimg(0), nokf, vimg(Tw - 2), kimg(0), vimg(0), pre, q, sA, sA,
                                                                 X.c, m, lim_of(Tw - 1), l, pB, pA, o);
        pv_tile(vimg(Tw - 1), pA, o);

        const bool bad = __builtin_amdgcn_ballot_w64(rvalid && !(l < kBig)) != 0;
        // the rest of the pass's staging, for the wavefronts whose blocks see further (before this
        // wavefront's store: they are the ones the pass is waiting for)
        for (t = t_own; t + 1 <= T - 2; t += 2) {
            stage_write(t + 2, kv0, vv0);
            stage_write(t + 3, kv1, vv1);
            cand_stage_load(g, t + 4, kv0, vv0);
            cand_stage_load(g, t + 5, kv1, vv1);
            __syncthreads();
        }
        store_block_rows(a, X, row, m, l, o);
        if (X.lane == 0)
            *(lds_int *)X.scr = bad ? 1 : 0;
        __syncthreads(); // ends the pass: the ring is free, the verdicts are visible
        wg_bad |= __builtin_amdgcn_ballot_w64(*(lds_int *)(smem + kRing * kSlotBytes + (X.lane & (kNW - 1)) * kScrBytes) !=
                                              0) != 0;
    }

    // The general sweep, as in the pipelined kernel above.
    if (wg_bad || wg_short)
        for (int p2 = blockIdx.x; p2 < npasses; p2 += gridDim.x) {
            const CandPass ps2 = make_cand_pass(a, cs, p2, npasses, wave);
            set_vhead(a, X, ps2.vh);
            if (ps2.exists && (wg_bad || (X.P + kTileKeys - 1) / kTileKeys < kMinTiles))
                general_pass(a, X, smem, tid, ps2.vh, ps2.blk, ps2.active);
        }
}

int device_cu_count(hipError_t &e)
{
    static DeviceSlots cu_by_device;
    return device_setup_once(cu_by_device, e, [] {
        hipError_t s = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_general_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (s == hipSuccess)
            s = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_pipelined_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (s == hipSuccess)
            s = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_pipelined_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (s == hipSuccess)
            s = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_candidate_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        return s;
    });
}

} // namespace

bool mfma_supported(const Args &a, int dtype)
{
    if (dtype != 1 || a.D != kD)
        return false;
    const long long rows = (long long)a.C * a.S * a.G;
    return rows <= 0x7fffffffLL - kPassRows && stream_pass_ids(a) <= 0x7fffffffLL - 8;
}

hipError_t launch_mfma(const Args &a, hipStream_t stream)
{
    // Suffix-side segments longer than one 32-key step (suffix, template and target together,
    // Sec. 3) go to the streamed kernel whenever its pipelined pass applies: it runs every
    // suffix step against the fixed reference, the resident kernels would fall back to their
    // general path for such shapes.
    const int max_tiles = (a.P + kTileKeys - 1) / kTileKeys;
    const bool long_suffix = a.S > kTileKeys && ((long long)a.S * a.G) % kBlockRows == 0 && max_tiles >= kMinTiles &&
                             (long long)a.P * a.kp_sp * 2 < 0x7fffffffLL;
    return resident_supported(a) && !long_suffix ? launch_resident(a, stream) : launch_stream(a, stream);
}

hipError_t launch_stream(const Args &a, hipStream_t stream)
{
    hipError_t e;
    const int num_cu = device_cu_count(e);
    if (e != hipSuccess)
        return e;
    const int max_tiles = (a.P + kTileKeys - 1) / kTileKeys;
    const long long npasses = stream_pass_ids(a);
    const unsigned grid = (unsigned)(npasses < num_cu ? npasses : num_cu);
    const bool pipelined = ((long long)a.S * a.G) % kBlockRows == 0 && max_tiles >= kMinTiles &&
                           (long long)a.P * a.kp_sp * 2 < 0x7fffffffLL && block_offsets_fit(a);
    // Long suffix-side segments whose candidates fill most of a workgroup's eight wavefronts
    // take the candidate passes.
    if (pipelined && a.S > kTileKeys && (long long)a.S * a.ks_ss * 2 < 0x7fffffffLL) {
        CandShape cs;
        const long long nblk_c = (long long)a.S * a.G / kBlockRows;
        cs.nblk_c = (int)nblk_c;
        cs.ngrp = (int)((nblk_c + kNW - 1) / kNW);
        // Full passes first; the last one takes what is left.  With up to four blocks left every
        // SIMD has at most one busy wavefront in it and the pass runs twice as fast.
        cs.bpp = cs.nblk_c < kNW ? cs.nblk_c : kNW;
        const long long units = (long long)a.B * a.Hkv;
        const long long cpasses = (units + 7) / 8 * 8 * cs.ngrp;
        if (nblk_c * 10 >= (long long)cs.ngrp * kNW * 6 && cpasses <= 0x7fffffffLL - 8) {
            const unsigned cgrid = (unsigned)(cpasses < num_cu ? cpasses : num_cu);
            return launch_kernel(stream_candidate_kernel, dim3(cgrid), dim3(kNW * 64), kLdsBytes, stream, a, (int)cpasses, cs);
        }
    }
    if (!pipelined)
        return launch_kernel(stream_general_kernel, dim3(grid), dim3(kNW * 64), kLdsBytes, stream, a, (int)npasses);
    else if (a.S <= kTileKeys)
        return launch_kernel(stream_pipelined_kernel<true>, dim3(grid), dim3(kNW * 64), kLdsBytes, stream, a, (int)npasses);
    else
        return launch_kernel(stream_pipelined_kernel<false>, dim3(grid), dim3(kNW * 64), kLdsBytes, stream, a, (int)npasses);
}

} // namespace pskv
