// Resident-prefix MFMA kernels of batched candidate-suffix attention for gfx950
// (bf16 tensors, head dim 128, prefix of at most 256 rows).
//
// One persistent workgroup per compute unit owns one KV head.  It copies that head's whole
// prefix K and V (the compact prefix cache of Sec. 4.2: one copy, never expanded over the
// candidates) into LDS once, and then its 8 wavefronts walk independently, without any
// further workgroup barrier, over 32-row blocks of the stacked query rows
//     r = (b*S + i)*G + g      (suffix-centric alignment, Sec. 4.3)
// of that head.  For each block a wavefront runs Eq. 2 over [prefix ; own suffix] with one
// online-softmax state per row: prefix tiles of 32 keys come from LDS, the candidate's own
// suffix K rows come straight from global memory and its V rows through a 4 KB per-wave
// scratch tile.
//
// Two kernels share this layout.  The general one handles any shape.  The pipelined one
// handles the common case in which every 32-row block lies inside one candidate and the
// suffix fits one 32-key step: it overlaps, inside each wavefront, the score product of the
// next tile (matrix cores) with the exponentials of the current one (vector ALU), requests
// everything it needs from global memory a full block ahead, and never branches on data.
// Operand layouts and the pieces shared with the streaming kernels are in pskv_mfma.hpp.
#include "pskv_mfma.hpp"

namespace pskv {
namespace {

constexpr int kMaxTiles = 8; // resident prefix: at most 256 keys

// Copies the prefix K/V of the current virtual head into the fragment-major LDS images (whole
// workgroup of 512 threads).  All global loads are issued before the first LDS write, so their
// latencies overlap.
__device__ inline void stage_prefix(const Args &a, const Ctx &X, int ntiles, lds_u8 *kimg, lds_u8 *vimg, int tid)
{
    // The thread's place in the images is worked out here, from a thread id the compiler cannot
    // trace back, and the staging registers are defined on every path: kept alive across the
    // block loops of the callers instead, these values would be spilled.
    asm volatile("" : "+v"(tid));
    const TileSlot t = make_tile_slot(tid);
    uintx4 kv[kMaxTiles] = {}, vv[kMaxTiles] = {};
#pragma unroll
    for (int kt = 0; kt < kMaxTiles; ++kt)
        if (kt < ntiles)
            load_tile_chunks(a, X, t, kt, kv[kt], vv[kt]);
#pragma unroll
    for (int kt = 0; kt < kMaxTiles; ++kt)
        if (kt < ntiles)
            write_tile_chunks(X, t, kt, kimg + kt * kTileBytes, vimg + kt * kTileBytes, tid, kv[kt], vv[kt]);
}

// max_tiles: tiles of the padded prefix length; it fixes the LDS layout for every instruction.
__device__ inline Ctx make_ctx(const Args &a, lds_u8 *smem, int max_tiles, int tid)
{
    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.Mtot = a.C * a.S * a.G;
    X.c = a.scale * kLog2e;
    X.k_lane = smem + X.lane * 16;
    X.v_lane = smem + max_tiles * kTileBytes + X.lane * 8;
    X.scr = smem + 2 * max_tiles * kTileBytes + __builtin_amdgcn_readfirstlane(tid >> 6) * kScrBytes;
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    return X;
}

// ------------------------------------------------------------------------------------------
// General path: one block, start to finish, nothing in flight across blocks.  Any shape:
// several candidates per block, suffixes longer than one step, no prefix at all.
// ------------------------------------------------------------------------------------------
__device__ __attribute__((always_inline)) void general_block(const Args &a, const Ctx &X, int ntiles, int blk)
{
    const int r0 = blk * kBlockRows;
    const Row row = decode_row(a, X, blk);
    const bool rvalid = row.rin && (int)row.ri < clamp_len(a, row.rlen);
    if (__builtin_amdgcn_ballot_w64(rvalid) == 0) {
        store_zero_block(a, X, r0, row);
        return;
    }
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

    for (int kt = 0; kt < ntiles; ++kt) // prefix part: every row sees every real prefix key
        prefix_tile_classic(X, X.k_lane + kt * kTileBytes, X.v_lane + kt * kTileBytes, X.P - kt * kTileKeys, q, st);
    suffix_classic(a, X, r0, row, q, st);
    store_block(a, X, r0, row, rvalid, st.m, st.l, st.o);
}

// Work distribution shared by both kernels.  A "virtual head" is one (instruction, KV head)
// pair; there are VH = Np*Hkv of them, each with its own prefix and its own C*S*G stacked
// rows.  The grid is per_vh * vh_slots workgroups: workgroup w serves virtual heads
// w % vh_slots, + vh_slots, ... (consecutive workgroup ids, one per XCD in turn, take
// consecutive KV heads) and, within each, a share w / vh_slots out of per_vh of the row blocks.
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void resident_general_kernel(Args a, int per_vh, int vh_slots, int max_tiles)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    Ctx X = make_ctx(a, smem, max_tiles, tid);
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int VH = a.Np * a.Hkv;
    for (int vh = blockIdx.x % vh_slots; vh < VH; vh += vh_slots) {
        set_vhead(a, X, vh);
        const int ntiles = (X.P + kTileKeys - 1) / kTileKeys;
        __syncthreads(); // every wavefront is done with the images of the virtual head before
        stage_prefix(a, X, ntiles, smem, smem + max_tiles * kTileBytes, tid);
        __syncthreads();
        for (int blk = (blockIdx.x / vh_slots) * kNW + wave; blk < nblocks; blk += per_vh * kNW)
            general_block(a, X, ntiles, blk);
    }
}

// ------------------------------------------------------------------------------------------
// Pipelined path.  Preconditions (checked by the launcher): S*G is a multiple of 32, so a
// 32-row block lies inside one candidate; S <= 32, so the suffix is one 32-key step; and the
// prefix has at least three tiles.
//
// Softmax without per-tile maxima: the first prefix tile fixes the row's reference maximum;
// later tiles take exp2 relative to it whatever their own maximum is (a larger score just gives
// a weight above one, which fp32 sums and bf16 weights hold at full relative precision).  If a
// row's sum ends up at or above kBig, the wavefront goes over all its blocks once more with
// the general path after its main loop (rare; kept out of the main loop so that it costs it no
// registers).
// ------------------------------------------------------------------------------------------
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void resident_pipelined_kernel(Args a, int per_vh, int vh_slots, int max_tiles)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    Ctx X = make_ctx(a, smem, max_tiles, tid);
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const int VH = a.Np * a.Hkv;
    auto kimg = [&](int t) { return X.k_lane + t * kTileBytes; };
    auto vimg = [&](int t) { return X.v_lane + t * kTileBytes; };

    // Candidate (within the instruction) and first suffix position of a block, from its index:
    // block blk covers rows [32*blk, 32*blk+31] of candidate 32*blk / (S*G).
    // A block whose first row is already past its candidate's length holds nothing but padding.
    auto block_cand = [&](int blk) { return (int)fdiv(fdiv(blk * kBlockRows, a.div_g), a.div_s); };
    auto block_i_lo = [&](int blk) { return (int)fdiv(blk * kBlockRows, a.div_g) - block_cand(blk) * a.S; };
    // Advance to the next block of this wavefront that has a valid row; blocks of pure padding
    // on the way are stored as zeros here and now.
    // Every wavefront takes one contiguous range of blocks, so that a candidate's suffix K/V, which
    // all of its blocks read, is fetched by one compute unit.  The workgroup's share of the virtual
    // head's blocks is cut into four parts, one per SIMD.  The two wavefronts of a SIMD (slots w and
    // w + 4) are not served alike: the one launched first wins the arbitration for the matrix cores
    // and gets through a block about a fifth faster, so it takes 7/12 of the SIMD's part and the
    // other one the rest; with equal shares the second one runs on alone for the last sixth of the
    // launch (measured: 14:10 beats 12:12 by 2-3 %, 13:11 and 15:9 lie between).
    const int wslot = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slice = blockIdx.x / vh_slots;
    const int wg_lo = (int)((long long)nblocks * slice / per_vh), wg_hi = (int)((long long)nblocks * (slice + 1) / per_vh);
    const int simd = wslot & 3;
    const int part_lo = wg_lo + (wg_hi - wg_lo) * simd / 4, part_hi = wg_lo + (wg_hi - wg_lo) * (simd + 1) / 4;
    const int split = part_lo + ((part_hi - part_lo) * 7 + 6) / 12;
    const int blk_lo = wslot < 4 ? part_lo : split, blk_hi = wslot < 4 ? split : part_hi;
    auto skip_padding = [&](int blk) {
        while (blk < blk_hi && block_i_lo(blk) >= len_uniform(a, X.cand0 + block_cand(blk))) {
            store_zero_block_rows(a, X, decode_block(a, X, blk, X.head, X.cand0));
            ++blk;
        }
        return blk;
    };

    for (int vh = blockIdx.x % vh_slots; vh < VH; vh += vh_slots) {
    set_vhead(a, X, vh);
    const int T = (X.P + kTileKeys - 1) / kTileKeys;

    // first block of this wavefront: request its row decode and Q before the prefix copy
    const int first_blk = blk_lo;
    bool any_bad = false;
    int blk = skip_padding(first_blk);
    BlockRows nxt = decode_block(a, X, blk < blk_hi ? blk : nblocks - 1, X.head, X.cand0);
    uintx4 q[8]; // this block's Q fragments until their last use, then the next block's
    load_q_block(a, X, nxt, q);

    __syncthreads(); // every wavefront is done with the images of the virtual head before
    stage_prefix(a, X, T, smem, smem + max_tiles * kTileBytes, tid);
    __syncthreads();

    if (T < 3) { // this instruction's prefix is too short for the pipeline: general path
        for (int b2 = first_blk; b2 < blk_hi; ++b2)
            general_block(a, X, T, b2);
        continue;
    }

    while (blk < blk_hi) {
        const BlockRows row = nxt;
        // the block's suffix step: keys 0..skmax of its candidate
        const int i_hi = (int)fdiv(blk * kBlockRows + kBlockRows - 1, a.div_g) - (row.b - X.cand0) * a.S;
        const int skmax = i_hi < row.len - 1 ? i_hi : row.len - 1;
        // Loads are retired in issue order, so what is needed last is requested first.
        uintx4 skf[8], svf[2][4];
        load_suffix_k_block(a, X, row.b, 0, skmax, skf);

        // ---- first prefix tile: scores, reference maximum ----
        floatx16 sA, sB; // raw scores of the current and of the next tile, roles alternating
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sA[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(X.k_lane + ks * 1024)), as_bf16x8(q[ks]),
                                                         sA, 0, 0, 0);
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

        // ---- pipeline over the prefix tiles: step t = scores of tile t+1, weights of tile t,
        //      value product of tile t-1 ----
        pipe_tile<true, false, false, false, false, true, true>(kimg(1), skf, vimg(0), kimg(2), vimg(0), pre, q, sA, sB,
                                                                X.c, m, 0, l, pA, pA, o);
        pipe_tile<true, false, true, true, false, true, true>(kimg(2), skf, vimg(0), kimg(3 < T ? 3 : T - 1), vimg(1), pre,
                                                              q, sB, sA, X.c, m, 0, l, pA, pB, o);
        int t = 2;
        for (; t + 1 <= T - 2; t += 2) {
            pipe_tile<true, false, true, false, false, true, true>(kimg(t + 1), skf, vimg(t - 1), kimg(t + 2), vimg(t), pre,
                                                                   q, sA, sB, X.c, m, 0, l, pB, pA, o);
            pipe_tile<true, false, true, false, false, true, true>(kimg(t + 2), skf, vimg(t), kimg(t + 3 < T ? t + 3 : T - 1),
                                                                   vimg(t + 1), pre, q, sB, sA, X.c, m, 0, l, pA, pB, o);
        }
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
        load_suffix_v_block(a, X, row.b, 0, skmax, svf); // one step ahead of its use
        // ---- last prefix tile: the "next scores" are the suffix scores, from the K registers ----
        pipe_tile<true, true, true, false, false, false, true>(kimg(0), skf, vimg(T - 2), kimg(0), vimg(T - 1), pre, q, sA,
                                                               sB, X.c, m, 0, l, pB, pA, o);

        // Q has been used for the last time: the next block's row decode and Q take its place.
        // (Requested unconditionally, for a clamped block index past the end: a load under a
        // branch would have to be waited for and copied at the join.)
        blk = skip_padding(blk + 1);
        nxt = decode_block(a, X, blk < blk_hi ? blk : nblocks - 1, X.head, X.cand0);
        load_q_block(a, X, nxt, q);

        // ---- suffix step: causal mask and weights under the value product of the last prefix
        //      tile; then the suffix value product through the scratch tile ----
        // the row sees keys 0..ri; element e holds key 8*(e/4) + e%4 + 4*h
        pipe_tile<false, false, true, false, true, false, false>(kimg(0), skf, vimg(T - 1), kimg(0), vimg(0), pre, q, sB, sB,
                                                                 X.c, m, (int)row.ri - 4 * X.h, l, pA, pB, o);
        pv_from_scratch(X, svf[0], as_bf16x8(pB[0]), o);
        pv_from_scratch(X, svf[1], as_bf16x8(pB[1]), o);

        any_bad |= __builtin_amdgcn_ballot_w64(row.ri < row.len && !(l < kBig)) != 0;
        store_block_rows(a, X, row, m, l, o);
    }

    // Rare: some row met scores far above its first tile's maximum.  Whatever this wavefront
    // stored is replaced by the general path's result.
    if (any_bad)
        for (int b2 = first_blk; b2 < blk_hi; ++b2)
            general_block(a, X, T, b2);
    } // virtual heads
}

} // namespace

bool resident_supported(const Args &a)
{
    return a.D == kD && a.P <= kMaxTiles * kTileKeys;
}

hipError_t launch_resident(const Args &a, hipStream_t stream)
{
    static DeviceSlots cu_by_device;
    hipError_t e;
    const int num_cu = device_setup_once(cu_by_device, e, [] {
        const int max_lds = 2 * kMaxTiles * kTileBytes + kNW * kScrBytes;
        hipError_t s = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_general_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (s == hipSuccess)
            s = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_pipelined_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        return s;
    });
    if (num_cu == 0)
        return e;
    const int max_tiles = (a.P + kTileKeys - 1) / kTileKeys;
    const long long rows = (long long)a.C * a.S * a.G; // stacked rows of one virtual head
    const long long nblocks = (rows + kBlockRows - 1) / kBlockRows;
    const long long VH = (long long)a.Np * a.Hkv;
    // One workgroup per compute unit.  With fewer virtual heads than compute units the
    // workgroups are split evenly over them (never more per virtual head than there are
    // groups of 8 row blocks); with more, every workgroup takes several in turn.
    const long long vh_slots = VH < num_cu ? VH : num_cu;
    long long per_vh = num_cu / vh_slots;
    const long long useful = (nblocks + kNW - 1) / kNW;
    if (per_vh > useful)
        per_vh = useful;
    const unsigned grid = (unsigned)(per_vh * vh_slots);
    const size_t lds = (size_t)2 * max_tiles * kTileBytes + kNW * kScrBytes;
    const bool pipelined = ((long long)a.S * a.G) % kBlockRows == 0 && a.S <= kTileKeys && max_tiles >= 3 &&
                           block_offsets_fit(a);
    if (pipelined)
        return launch_kernel(resident_pipelined_kernel, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_vh,
                           (int)vh_slots, max_tiles);
    else
        return launch_kernel(resident_general_kernel, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_vh,
                           (int)vh_slots, max_tiles);
}

} // namespace pskv
