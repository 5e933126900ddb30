// Matrix-core kernel for the query gradient of batched candidate-suffix attention on gfx950
// (bf16 tensors, head dim 128, prefix of any length - one shared prefix or one per instruction of
// the batched multi-instruction form -, any suffix shape).
//
// For a query row with softmax weights p_j = exp(s_j - lse) over its visible rows
// (prefix, then own suffix rows 0..i; derivative of Eq. 2, prefix K/V constant):
//     dp_j = <dout_row, V_j>,   ds_j = p_j (dp_j - <dout_row, out_row>),   dq_row = scale * sum_j ds_j K_j.
// Work is laid out as in the streamed forward kernels: a pass is one (KV head, group of 256
// stacked rows r = (b*S + i)*G + g) pair, each of the 8 wavefronts of a workgroup owns one
// 32-row block, and the prefix goes through LDS tile by tile (32 keys), double-buffered, one
// barrier per tile, read from HBM once and used by all 256 rows.  Per tile and block, with the
// transposed formulation of pskv_mfma.hpp (a lane owns one query column):
//     S^T  = K Q^T        A = K fragment (row-major image),   B = Q fragment
//     dP^T = V dO^T       A = V fragment (row-major image),   B = dO fragment
//     dS^T = P^T o (dP^T - D)                                 vector ALU, P^T = exp2(c S^T - lse)
//     dQ^T += K^T dS^T    A = K^T fragment (transposing image), B = dS^T packed to bf16
// so a slot of the LDS ring holds three 8 KB images: K and V row-major, K once more in the
// layout the transposing read wants.  The suffix rows of the block's own candidate(s) follow,
// with K/V fragments straight from global memory and K^T through the per-wave scratch tile.
// No running maximum is needed: lse comes from the forward pass, every weight is at most one.
// A second kernel further down keeps short prefixes resident in LDS instead of streaming them.
#include "pskv_mfma.hpp"
#include <type_traits>

// Scratch of the entry point that allocates nothing (pskv_attn_bwd_noalloc): <dout_row, out_row> of
// every query row, B*Hq*S floats, handed from the dq kernel to the dk/dv kernel.  In host code this
// name is a stand-in for the symbol, not a device address: the address comes from
// hipGetSymbolAddress (noalloc_scratch() at the end of this file) and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[pskv::kNoAllocScratchBytes];

namespace pskv {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBwdSlotBytes = 3 * kTileBytes;
constexpr int kBwdLdsBytes = 2 * kBwdSlotBytes + kNW * kScrBytes;
constexpr int kBwdPassRows = kNW * kBlockRows;

// Rows of a [.,.,H,D] tensor laid out like out (dout, out): lane (row c32, half h) gets
// d = 16*ks + 8*h ..+7 for ks = 0..7, as load_q does for q.
__device__ inline void load_o_like(const Args &a, const Ctx &X, const Row &x, const void *base, uintx4 (&dst)[8])
{
    const unsigned short *r = reinterpret_cast<const unsigned short *>(base) + (long long)x.rb * a.o_sb +
                              (long long)x.ri * a.o_ss + (long long)x.rh * a.o_sh + 8 * X.h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        dst[ks] = ld_global16(r + 16 * ks);
}

// Where <dout_row, out_row> of query row (candidate b, query head rh, suffix position ri) sits in
// the workspace: in the order of the stacked rows of its KV head, ((b*Hkv + k)*S + ri)*G + g, so
// that the 32 rows of a block are 128 contiguous bytes for the kernel that writes them and for
// the one that reads them back.
__device__ inline long long delta_index(const Args &a, long long b, int rh, int ri)
{
    const int k = (int)fdiv((unsigned)rh, a.div_g), gq = rh - k * a.G;
    return ((b * a.Hkv + k) * a.S + ri) * a.G + gq;
}

__device__ inline float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }

// <dout_row, out_row> of the lane's row from the row's fragments (lane half h holds columns
// 16*ks + 8*h ..+7 of fragment ks).  Columns 0..63 and 64..127 are summed separately, each across the
// two lane halves, and then added: the order in which the dk/dv kernel, whose wavefronts hold one
// half of the columns each, forms the same number when no workspace hands it over - the two agree
// to the bit.
__device__ inline float half_dot(const uintx4 (&x)[8], const uintx4 (&y)[8], int half)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = __builtin_fmaf(bf16_lo(x[4 * half + i][e]), bf16_lo(y[4 * half + i][e]), acc);
            acc = __builtin_fmaf(bf16_hi(x[4 * half + i][e]), bf16_hi(y[4 * half + i][e]), acc);
        }
    return acc + __shfl_xor(acc, 32, 64);
}
__device__ inline float dout_dot_out(const uintx4 (&dof)[8], const uintx4 (&of)[8])
{
    return half_dot(dof, of, 0) + half_dot(dof, of, 1);
}

// dS^T of one 32-key tile from its raw scores s and dp; element e is visible iff vis(e).
// Returns the two B fragments (keys 0..15, 16..31) of the following product.
template <typename VIS>
__device__ inline void ds_tile(const floatx16 &s, const floatx16 &dp, float c, float lse2, float drow, VIS vis,
                               bf16x8 (&pf)[2])
{
    float ds[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float p = vis(e) ? fast_exp2(__builtin_fmaf(s[e], c, -lse2)) : 0.f;
        ds[e] = p * (dp[e] - drow);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        uintx4 w = {pack_bf16(ds[8 * j + 0], ds[8 * j + 1]), pack_bf16(ds[8 * j + 2], ds[8 * j + 3]),
                    pack_bf16(ds[8 * j + 4], ds[8 * j + 5]), pack_bf16(ds[8 * j + 6], ds[8 * j + 7])};
        pf[j] = as_bf16x8(w);
    }
}

// O^T-style accumulation for the 16-key step j of a 32-key tile whose rows the lanes hold as
// row-major fragments (lane (key c32, half h): columns 16*ks + 8*h ..+7 in frag[ks]): the lanes
// that own keys of step j put their chunks where the scratch image wants them - chunk (key r,
// columns 16*ks + 8*h) belongs to fragment (dt = ks/2, u = (r/8)%2), slot pair
// 16*((r/4)%2) + 8*(ks%2) + 2*(r%4) + h - and the transposing reads hand them back as A
// fragments (cf. pv_from_scratch, which takes the rows in image order from global memory).
__device__ inline void pv_from_fragments(const Ctx &X, const uintx4 (&frag)[8], int j, bf16x8 pfj, floatx16 (&o)[4])
{
    if ((X.c32 >> 4) == j) {
        const int u = (X.c32 >> 3) & 1;
        lds_u8 *dst = X.scr + u * 512 + (16 * ((X.c32 >> 2) & 1) + 2 * (X.c32 & 3) + X.h) * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            *(lds_u128 *)(dst + (ks >> 1) * 1024 + (ks & 1) * 128) = frag[ks];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    bf16x8 va[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        short4v lo = lds_read_tr(X.scr + X.lane * 8 + (dt * 2 + 0) * 512);
        short4v hi = lds_read_tr(X.scr + X.lane * 8 + (dt * 2 + 1) * 512);
        short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        __builtin_memcpy(&va[dt], &v8, 16);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt], pfj, o[dt], 0, 0, 0);
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void bwd_dq_mfma_kernel(BwdArgs g, int npasses)
{
    const Args &a = g.f;
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.Mtot = a.C * a.S * a.G;
    X.c = a.scale * kLog2e;
    X.k_lane = smem + X.lane * 16;                  // K row-major image of slot 0
    X.v_lane = smem + 2 * kTileBytes + X.lane * 8;  // K transposing image of slot 0
    X.scr = smem + 2 * kBwdSlotBytes + wave * kScrBytes;
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    lds_u8 *vk_lane = smem + kTileBytes + X.lane * 16; // V row-major image of slot 0
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const TileSlot t = make_tile_slot(tid);
    const int VH = a.Np * a.Hkv;
    // the gradient goes out through the forward pass's store routine: dq is laid out like q
    Args ad = a;
    ad.out = g.dq;
    ad.lse = nullptr;
    ad.o_sb = a.q_sb;
    ad.o_ss = a.q_ss;
    ad.o_sh = a.q_sh;

    for (int p = blockIdx.x; p < npasses; p += gridDim.x) {
        set_vhead(a, X, p % VH);
        const int blk_raw = (p / VH) * kNW + wave;
        const bool active = blk_raw < nblocks;
        const int blk = active ? blk_raw : nblocks - 1;
        const int r0 = blk * kBlockRows;
        const int ntiles = (X.P + kTileKeys - 1) / kTileKeys;
        const Row row = decode_row(a, X, blk);
        const bool rvalid = active && row.rin && (int)row.ri < clamp_len(a, row.rlen);
        const bool work = __builtin_amdgcn_ballot_w64(rvalid) != 0;

        // requested first, so that it is there with the rows below and costs no round trip of its own
        const float lse2 = (row.rin ? a.lse[((long long)row.rb * a.Hq + row.rh) * a.S + row.ri] : 0.f) * kLog2e;
        // Rows past their candidate's length take the data of its last position (never fetched
        // otherwise): what they compute is finite and stored as zero.
        Row rld = row;
        {
            const int len = clamp_len(a, row.rlen);
            rld.ri = (int)row.ri < len ? row.ri : (len > 0 ? (unsigned)(len - 1) : 0u);
        }
        uintx4 q[8], dof[8];
        load_q(a, X, rld, q);
        load_o_like(a, X, rld, g.dout, dof);
        float drow; // <dout_row, out_row>
        {
            uintx4 of[8];
            load_o_like(a, X, rld, a.out, of);
            drow = dout_dot_out(dof, of);
        }
        if (g.delta && rvalid && X.h == 0) // kept in the order of the stacked rows: see delta_index
            g.delta[delta_index(a, row.rb, row.rh, row.ri)] = drow;

        floatx16 o[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                o[dt][e] = 0.f;

        // ---- prefix part: every row sees every prefix key ----
        if (ntiles > 0) {
            uintx4 kk, vk, kt2;
            auto fetch = [&](int kt) {
                uintx4 unused;
                load_tile_chunks(a, X, t, kt, kk, unused);   // K chunk for the row-major image; (V chunk of the transposing slot unused)
                // V chunk for the row-major image and K chunk for the transposing image
                const int last = X.P > 0 ? X.P - 1 : 0;
                const int kkey = kt * kTileKeys + t.k_row, vkey = kt * kTileKeys + t.v_row;
                vk = ld_global16(X.vpg + (long long)(kkey < X.P ? kkey : last) * a.kp_sp + t.k_chunk * 8);
                kt2 = ld_global16(X.kpg + (long long)(vkey < X.P ? vkey : last) * a.kp_sp + t.v_chunk * 8);
            };
            auto put = [&](int kt, int slot) {
                const int kkey = kt * kTileKeys + t.k_row, vkey = kt * kTileKeys + t.v_row;
                lds_u8 *s0 = smem + slot * kBwdSlotBytes + tid * 16;
                *(lds_u128 *)s0 = kkey < X.P ? kk : uintx4{0, 0, 0, 0};
                *(lds_u128 *)(s0 + kTileBytes) = kkey < X.P ? vk : uintx4{0, 0, 0, 0};
                *(lds_u128 *)(s0 + 2 * kTileBytes) = vkey < X.P ? kt2 : uintx4{0, 0, 0, 0};
            };
            fetch(0);
            __syncthreads(); // whatever the slots held has been used by every wavefront
            put(0, 0);
            __syncthreads();
            for (int kt = 0; kt < ntiles; ++kt) {
                fetch(kt + 1 < ntiles ? kt + 1 : kt);
                if (work) {
                    const int so = (kt & 1) * kBwdSlotBytes;
                    floatx16 s, dp;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        s[e] = 0.f;
                        dp[e] = 0.f;
                    }
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(X.k_lane + so + ks * 1024)),
                                                                    as_bf16x8(q[ks]), s, 0, 0, 0);
                        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(vk_lane + so + ks * 1024)),
                                                                     as_bf16x8(dof[ks]), dp, 0, 0, 0);
                    }
                    const int nv = X.P - kt * kTileKeys - 4 * X.h; // element e holds key 8*(e/4) + e%4 + 4*h of the tile
                    bf16x8 pf[2];
                    if ((kt + 1) * kTileKeys <= X.P) // a full tile: every row sees all of it
                        ds_tile(s, dp, X.c, lse2, drow, [](int) { return true; }, pf);
                    else
                        ds_tile(s, dp, X.c, lse2, drow, [&](int e) { return 8 * (e >> 2) + (e & 3) < nv; }, pf);
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int dt = 0; dt < 4; ++dt)
                            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_fragment(X.v_lane + so, dt, j), pf[j], o[dt], 0,
                                                                            0, 0);
                }
                if (kt + 1 < ntiles)
                    put(kt + 1, (kt + 1) & 1);
                __syncthreads();
            }
        }

        // ---- suffix part: (candidate, 32-key step) pairs, wave-uniform ----
        if (work) {
            Ctx Xs = X; // the suffix V rows are fetched as row-major fragments too: the K loader pointed at V
            Xs.ksg = X.vsg;
            const int last_row = r0 + kBlockRows - 1 < X.Mtot ? r0 + kBlockRows - 1 : X.Mtot - 1;
            const int tok_first = fdiv(r0, a.div_g), tok_last = fdiv(last_row, a.div_g);
            const int bl_last = fdiv(tok_last, a.div_s);
            for (int bl = fdiv(tok_first, a.div_s); bl <= bl_last; ++bl) {
                const int b = X.cand0 + bl;
                const int len = len_uniform(a, b);
                const int i_lo = tok_first - bl * a.S > 0 ? tok_first - bl * a.S : 0;
                const int i_hi = tok_last - bl * a.S < a.S - 1 ? tok_last - bl * a.S : a.S - 1;
                const int kmax = i_hi < len - 1 ? i_hi : len - 1;
                if (i_lo >= len)
                    continue;
                for (int k0 = 0; k0 <= kmax; k0 += kTileKeys) {
                    floatx16 s, dp;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        s[e] = 0.f;
                        dp[e] = 0.f;
                    }
                    // K rows once, as row-major fragments: A operands of S^T here, and the source of the
                    // transposed fragments of dQ^T further down
                    uintx4 kf[8];
                    load_suffix_k(a, X, b, k0, kmax, kf);
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks)
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), as_bf16x8(q[ks]), s, 0, 0, 0);
                    {
                        uintx4 vf[8];
                        load_suffix_k(a, Xs, b, k0, kmax, vf); // V rows as row-major fragments
#pragma unroll
                        for (int ks = 0; ks < 8; ++ks)
                            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vf[ks]), as_bf16x8(dof[ks]), dp, 0, 0, 0);
                    }
                    // the row sees keys 0..ri of its own candidate; element e holds key k0 + 8*(e/4) + e%4 + 4*h
                    const int lim = ((int)row.rb == b ? (int)row.ri : -1) - k0 - 4 * X.h;
                    bf16x8 pf[2];
                    ds_tile(s, dp, X.c, lse2, drow, [&](int e) { return 8 * (e >> 2) + (e & 3) <= lim; }, pf);
                    pv_from_fragments(X, kf, 0, pf[0], o);
                    pv_from_fragments(X, kf, 1, pf[1], o);
                }
            }
        }
        if (active) {
            if (work) // store_block divides by the sum of both half-waves' l: 1/(2 * 0.5/scale) = scale
                store_block(ad, X, r0, row, rvalid, 0.f, 0.5f / a.scale, o);
            else
                store_zero_block(ad, X, r0, row);
        }
    }
}

// ------------------------------------------------------------------------------------------
// dq with the prefix resident in LDS (prefix of at most 256 rows, every 32-row block inside one
// candidate): the layout of work of the resident forward kernel.  A persistent workgroup copies
// the prefix K and V of its (instruction, KV head) pair into LDS once; its eight wavefronts
// then walk independently, without any further workgroup barrier, over the pair's 32-row blocks.
//
// Two 8 KB images per 32-key tile serve the three products.  V is kept as row-major fragments
// (the "K image" layout of pskv_mfma.hpp) for dP^T = V dO^T.  K is kept once, in the
// transposable layout (the "V image" layout), from which K^T dS^T takes its A fragments through
// the transposing read; S^T = K Q^T needs row-major K fragments, and the 16 bytes a lane wants
// for those are two neighbouring 8-byte slots of that same image.  Read that way the lanes of a
// quarter-wave would hit only a quarter of the banks, so the 16-byte chunks of each 512-byte
// fragment are stored permuted, chunk p at p ^ (p >> 4) ^ 8u (u: the fragment's 8-key half), which
// makes both kinds of read conflict-free: lanes pay with one precomputed address per kind.
// ------------------------------------------------------------------------------------------
constexpr int kDqMaxTiles = 8;

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void bwd_dq_resident_kernel(BwdArgs g, int per_vh, int vh_slots, int max_tiles)
{
    const Args &a = g.f;
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.Mtot = a.C * a.S * a.G;
    X.c = a.scale * kLog2e;
    lds_u8 *vrm = smem;                             // V images, row-major fragments
    lds_u8 *ktr = smem + max_tiles * kTileBytes;    // K images, transposable, chunks permuted
    X.k_lane = vrm + X.lane * 16;
    X.v_lane = ktr + X.lane * 8; // not used for reads (see k_rm and k_tr below)
    X.scr = smem + 2 * max_tiles * kTileBytes + wave * kScrBytes;
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    // Row-major K fragment of contraction step ks for key c32, half h: logical chunk
    // 16*hk + 8*(ks%2) + 2*(key%4) + h of fragment (dt = ks/2, j, u); hk, u, j are bits 2, 3, 4 of the key.
    const int hk = (X.c32 >> 2) & 1, uk = (X.c32 >> 3) & 1, jk = X.c32 >> 4;
    const int k_rm_common = jk * 1024 + uk * 512 + (16 * hk + 2 * (X.c32 & 3) + (X.h ^ hk)) * 16;
    lds_u8 *k_rm[2] = {ktr + k_rm_common + 8 * uk * 16, ktr + k_rm_common + 8 * (1 - uk) * 16}; // even ks, odd ks
    // Transposing read of fragment (dt, j, u): this lane's slot l sits in chunk (l >> 1) ^ (l >> 5) ^ 8u.
    lds_u8 *k_tr[2] = {ktr + (((X.lane >> 1) ^ X.h) * 16 + (X.lane & 1) * 8),
                       ktr + (((X.lane >> 1) ^ X.h ^ 8) * 16 + (X.lane & 1) * 8)};
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const int blk_stride = per_vh * kNW;
    const int VH = a.Np * a.Hkv;
    // the gradient goes out through the forward pass's store routine: dq is laid out like q
    Args ad = a;
    ad.out = g.dq;
    ad.lse = nullptr;
    ad.o_sb = a.q_sb;

    for (int vh = blockIdx.x % vh_slots; vh < VH; vh += vh_slots) {
        set_vhead(a, X, vh);
        const int T = (X.P + kTileKeys - 1) / kTileKeys;
        __syncthreads(); // every wavefront is done with the images of the virtual head before
        { // four tiles at a time: more would not fit the register file next to what the block loop keeps
            // The thread's place in the images is worked out here, from a thread id the compiler
            // cannot trace back: kept across the block loop instead, these values would be spilled.
            int tid_here = tid;
            asm volatile("" : "+v"(tid_here));
            const TileSlot t = make_tile_slot(tid_here);
            const int last = X.P > 0 ? X.P - 1 : 0;
            const int fr = tid_here >> 5, p5 = tid_here & 31;
            const int pos = p5 ^ (p5 >> 4) ^ (8 * (fr & 1));
#pragma unroll
            for (int kt0 = 0; kt0 < kDqMaxTiles; kt0 += 4) {
                uintx4 vk[4] = {}, kk[4] = {}; // defined on every path: nothing of them outlives the iteration
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (kt0 + i < T) {
                        const int kkey = (kt0 + i) * kTileKeys + t.k_row, vkey = (kt0 + i) * kTileKeys + t.v_row;
                        vk[i] = ld_global16(X.vpg + (long long)(kkey < X.P ? kkey : last) * a.kp_sp + t.k_chunk * 8);
                        kk[i] = ld_global16(X.kpg + (long long)(vkey < X.P ? vkey : last) * a.kp_sp + t.v_chunk * 8);
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (kt0 + i < T) {
                        const int kt = kt0 + i;
                        const int kkey = kt * kTileKeys + t.k_row, vkey = kt * kTileKeys + t.v_row;
                        *(lds_u128 *)(vrm + kt * kTileBytes + tid_here * 16) = kkey < X.P ? vk[i] : uintx4{0, 0, 0, 0};
                        *(lds_u128 *)(ktr + kt * kTileBytes + fr * 512 + pos * 16) = vkey < X.P ? kk[i] : uintx4{0, 0, 0, 0};
                    }
            }
        }
        __syncthreads();

        for (int blk = (blockIdx.x / vh_slots) * kNW + wave; blk < nblocks; blk += blk_stride) {
            const BlockRows row = decode_block(a, X, blk, X.head, X.cand0);
            // where the lane's row sits in dq (laid out like q), as store_block_rows wants it
            BlockRows rowd = row;
            rowd.o_off = ((unsigned)row.ri * (unsigned)a.q_ss + (unsigned)row.rh * (unsigned)a.q_sh) * 2u;
            const int i_lo = (int)fdiv(blk * kBlockRows, a.div_g) - (row.b - X.cand0) * a.S;
            if (i_lo >= row.len) { // nothing but padding
                store_zero_block_rows(ad, X, rowd);
                continue;
            }
            const int i_hi = (int)fdiv(blk * kBlockRows + kBlockRows - 1, a.div_g) - (row.b - X.cand0) * a.S;
            const int kmax = i_hi < row.len - 1 ? i_hi : row.len - 1;

            // requested first, so that it is there with the rows below and costs no round trip of its own
            const float lse2 = a.lse[((long long)row.b * a.Hq + row.rh) * a.S + row.ri] * kLog2e;
            uintx4 q[8], dof[8];
            load_q_block(a, X, row, q);
            float drow; // <dout_row, out_row>
            {
                // rows past the candidate's length take dout and out of its last position, as they do for q
                const int rld = row.ri < row.len ? row.ri : row.len - 1;
                const unsigned ld_off = ((unsigned)rld * (unsigned)a.o_ss + (unsigned)row.rh * (unsigned)a.o_sh) * 2u;
                const long long obase = (long long)row.b * a.o_sb * 2;
                const unsigned char *dorow = reinterpret_cast<const unsigned char *>(g.dout) + obase + (ld_off + 16u * X.h);
                const unsigned char *orow = reinterpret_cast<const unsigned char *>(a.out) + obase + (ld_off + 16u * X.h);
                uintx4 of[8];
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    dof[ks] = *reinterpret_cast<const uintx4 *>(dorow + 32 * ks);
                    of[ks] = *reinterpret_cast<const uintx4 *>(orow + 32 * ks);
                }
                drow = dout_dot_out(dof, of);
            }
            if (g.delta && row.ri < row.len && X.h == 0) // one 128-byte line per block: see delta_index
                g.delta[delta_index(a, row.b, row.rh, row.ri)] = drow;

            floatx16 o[4];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    o[dt][e] = 0.f;

            // ---- prefix part: every row sees every prefix key (only a ragged last tile has keys to hide) ----
            auto prefix_tile = [&](int kt, auto ragged) {
                const int to = kt * kTileBytes;
                floatx16 s, dp;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    s[e] = 0.f;
                    dp[e] = 0.f;
                }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(k_rm[ks & 1] + to + (ks >> 1) * 2048)),
                                                                as_bf16x8(q[ks]), s, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(X.k_lane + to + ks * 1024)),
                                                                 as_bf16x8(dof[ks]), dp, 0, 0, 0);
                }
                const int nv = X.P - kt * kTileKeys - 4 * X.h; // element e holds key 8*(e/4) + e%4 + 4*h of the tile
                bf16x8 pf[2];
                if constexpr (decltype(ragged)::value)
                    ds_tile(s, dp, X.c, lse2, drow, [&](int e) { return 8 * (e >> 2) + (e & 3) < nv; }, pf);
                else
                    ds_tile(s, dp, X.c, lse2, drow, [](int) { return true; }, pf);
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        short4v lo = lds_read_tr(k_tr[0] + to + ((dt * 2 + j) * 2 + 0) * 512);
                        short4v hi = lds_read_tr(k_tr[1] + to + ((dt * 2 + j) * 2 + 1) * 512);
                        short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        bf16x8 kf;
                        __builtin_memcpy(&kf, &v8, 16);
                        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, pf[j], o[dt], 0, 0, 0);
                    }
            };
            const int Tfull = X.P / kTileKeys;
            for (int kt = 0; kt < Tfull; ++kt)
                prefix_tile(kt, std::false_type{});
            if (Tfull < T)
                prefix_tile(Tfull, std::true_type{});

            // ---- suffix part: 32-key steps of the block's own candidate ----
            {
                Ctx Xs = X; // the suffix V rows are fetched as row-major fragments too: the K loader pointed at V
                Xs.ksg = X.vsg;
                for (int k0 = 0; k0 <= kmax; k0 += kTileKeys) {
                    floatx16 s, dp;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        s[e] = 0.f;
                        dp[e] = 0.f;
                    }
                    // K rows once, as row-major fragments: A operands of S^T here, and the source of the
                    // transposed fragments of dQ^T further down
                    uintx4 kf[8];
                    load_suffix_k_block(a, X, row.b, k0, kmax, kf);
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks)
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), as_bf16x8(q[ks]), s, 0, 0, 0);
                    {
                        uintx4 vf[8];
                        load_suffix_k_block(a, Xs, row.b, k0, kmax, vf); // V rows as row-major fragments
#pragma unroll
                        for (int ks = 0; ks < 8; ++ks)
                            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vf[ks]), as_bf16x8(dof[ks]), dp, 0, 0, 0);
                    }
                    // the row sees keys 0..ri of its candidate; element e holds key k0 + 8*(e/4) + e%4 + 4*h
                    const int lim = row.ri - k0 - 4 * X.h;
                    bf16x8 pf[2];
                    ds_tile(s, dp, X.c, lse2, drow, [&](int e) { return 8 * (e >> 2) + (e & 3) <= lim; }, pf);
                    pv_from_fragments(X, kf, 0, pf[0], o);
                    pv_from_fragments(X, kf, 1, pf[1], o);
                }
            }
            // store_block_rows divides by the sum of both half-waves' l: 1/(2 * 0.5/scale) = scale
            store_block_rows(ad, X, rowd, 0.f, 0.5f / a.scale, o);
        }
    }
}

// ------------------------------------------------------------------------------------------
// dk_suf, dv_suf on the matrix cores.  One workgroup of two wavefronts per (candidate, KV head, tile
// of 32 suffix keys); wavefront DH owns half DH of the 128 columns (the accumulators of both halves
// would not fit one register file).  The pair walks over the candidate's 32-row blocks of stacked
// query rows (i, g) that can see the tile and accumulates, in the non-transposed formulation (a lane
// owns one key column):
//     S   = Q K^T          A = Q fragment,   B = K fragment (both straight from global memory)
//     dP  = dO V^T         A = dO fragment,  B = V fragment
//     P   = exp2(c S - lse),  dS = P o (dP - D)      per element: row quantities come through LDS
//     dV^T += dO^T P       A = dO^T through the scratch tile,  B = P packed to bf16
//     dK^T += Q^T dS       A = Q^T through the scratch tile,   B = dS packed to bf16
// The first two products contract over the 128 columns: each wavefront forms its own half of that
// sum from its own half of the columns of q, dout, K and V - the only columns it ever fetches, so
// that every row of q and dout crosses HBM once per tile and not once per wavefront - and the
// halves change hands through LDS: a wavefront completes S and dP, and takes the exponentials,
// for one of the block's two 16-row steps only (it receives the other wavefront's half of the
// sums for those rows, 2 KB each of S and dP in fp32) and passes that step's packed P and dS on
// to the other one.  The second products need exactly the columns the wavefront already holds.
// The accumulators of S hold, for lane half h, rows 8*kk + 4*h + t of the block in element
// 4*kk + t: exactly the order in which the scratch image hands out the rows of dO and Q, so P
// and dS go from the first products to the second ones through registers only.
// ------------------------------------------------------------------------------------------
constexpr int kDkvWaves = 2; // the two column halves of one unit
constexpr int kDkvScrBytes = 4 * 2048; // per wavefront: the four images dO and Q are transposed through (the first 4 KB also
                                       // serve the final store)
constexpr int kDkvAux = 512; // per wavefront: lse, <dout,out> and suffix position of the block's 32 rows
constexpr int kDkvXchBytes = 2 * 8 * 256 + 2 * 1024; // per wavefront, for the other one: its halves of S and dP for that one's
                                                     // 16-row step (8 accumulator registers of 256 bytes each), then its own
                                                     // step's packed weights and score gradients
constexpr int kDkvLdsBytes = kDkvWaves * (kDkvScrBytes + kDkvAux + kDkvXchBytes) + 256; // + the halves of <dout,out>

// dO^T and Q^T of a 32-row block as A operands of the second products, from the row-major
// fragments the lanes hold for the first ones (lane (row c32, half h): columns 16*i + 8*h ..+7 of
// this wavefront's 64 in frag[i]).  Each lane puts its chunks where a scratch image wants them -
// four images of 2 KB, one per (16-row step j, tensor): chunk (row r, columns 16*i + 8*h) belongs
// to fragment (i/2, u = (r/8)%2), slot pair 16*((r/4)%2) + 8*(i%2) + 2*(r%4) + h - and the
// transposing reads hand them back: at[j][w][i2] is the A fragment of step j, tensor w (0: dO,
// 1: Q), 32-column group i2 of the wavefront's half.  All of it is written, then all of it read:
// nothing here depends on the weights, so the whole exchange runs under the first products.
__device__ inline void transpose_halves(const Ctx &X, const uintx4 (&doh)[4], const uintx4 (&qh)[4], bf16x8 (&at)[2][2][2])
{
    const int j = X.c32 >> 4, u = (X.c32 >> 3) & 1;
    lds_u8 *dst = X.scr + j * 4096 + u * 512 + (16 * ((X.c32 >> 2) & 1) + 2 * (X.c32 & 3) + X.h) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        *(lds_u128 *)(dst + (i >> 1) * 1024 + (i & 1) * 128) = doh[i];
        *(lds_u128 *)(dst + 2048 + (i >> 1) * 1024 + (i & 1) * 128) = qh[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const lds_u8 *img = X.scr + (2 * jj + w) * 2048 + X.lane * 8;
                short4v lo = lds_read_tr(const_cast<lds_u8 *>(img) + (i2 * 2 + 0) * 512);
                short4v hi = lds_read_tr(const_cast<lds_u8 *>(img) + (i2 * 2 + 1) * 512);
                short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                __builtin_memcpy(&at[jj][w][i2], &v8, 16);
            }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int DH, bool HAS_DELTA>
__device__ __attribute__((always_inline)) void bwd_dkv_unit(const BwdArgs &g, lds_u8 *smem, int tid, int bk, int kt)
{
    const Args &a = g.f;
    const int k = bk % a.Hkv, b = bk / a.Hkv;
    const int k0 = kt * kTileKeys;

    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.Mtot = a.S * a.G; // rows of this candidate
    X.c = a.scale * kLog2e;
    X.scr = smem + DH * (kDkvScrBytes + kDkvAux);
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    X.head = k;
    X.cand0 = 0;
    X.P = 0;
    X.ksg = reinterpret_cast<const unsigned short *>(a.ks) + (long long)k * a.ks_sh;
    X.vsg = reinterpret_cast<const unsigned short *>(a.vs) + (long long)k * a.ks_sh;
    typedef __attribute__((address_space(3))) float lds_f32;
    typedef __attribute__((address_space(3))) floatx4 lds_f32x4;
    lds_f32 *aux_lse = (lds_f32 *)(X.scr + kDkvScrBytes);
    lds_f32 *aux_drow = aux_lse + 32;
    lds_f32 *aux_i = aux_drow + 32; // suffix position of the row as a float, -1 for a row that does not count
    // where the halves of S and dP change hands: mine to write, the other wavefront's to read
    lds_u8 *xch = smem + kDkvWaves * (kDkvScrBytes + kDkvAux);
    lds_u8 *xch_mine = xch + DH * kDkvXchBytes + X.lane * 16, *xch_other = xch + (1 - DH) * kDkvXchBytes + X.lane * 16;
    lds_f32 *xdrow = (lds_f32 *)(xch + kDkvWaves * kDkvXchBytes); // [2][32]: the halves of <dout,out>

    const int len = len_uniform(a, b);
    const int key = k0 + X.c32; // this lane's key
    floatx16 dk[2], dv[2]; // output columns 64*DH .. 64*DH+63
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            dk[dt][e] = 0.f;
            dv[dt][e] = 0.f;
        }

    if (k0 < len) { // the same for both wavefronts of the workgroup: the barriers below are met by both
        const int kmax = len - 1;
        const unsigned short *qb = reinterpret_cast<const unsigned short *>(a.q) + (long long)b * a.q_sb + (long long)k * a.G * a.q_sh;
        const long long ob = (long long)b * a.o_sb + (long long)k * a.G * a.o_sh;
        const unsigned short *dob = reinterpret_cast<const unsigned short *>(g.dout) + ob;
        const unsigned short *outb = reinterpret_cast<const unsigned short *>(a.out) + ob;
        const int nrows = len * a.G; // rows (i, g) with i < len, in stacked order i*G + g
        // this half's columns of the tile's K and V rows as row-major fragments (rows past kmax clamped:
        // never visible): the same for every block of rows
        uintx4 kfh[4], vfh[4];
        {
            const int krow = k0 + X.c32 < kmax ? k0 + X.c32 : kmax;
            const long long koff = (long long)b * a.ks_sb + (long long)krow * a.ks_ss + 8 * X.h + 64 * DH;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kfh[i] = ld_global16(X.ksg + koff + 16 * i);
                vfh[i] = ld_global16(X.vsg + koff + 16 * i);
            }
        }
        // What a block needs from global memory, all requested in one round trip: this half's columns
        // of q and dout (kept for the second products) and the row quantities of this lane's row of
        // the block, clamped into the candidate.
        struct BlockIn {
            uintx4 qh[4], doh[4];
            float lse_row, drow;
            int ri;
            bool rvalid;
        };
        auto fetch = [&](int rl0, BlockIn &x, uintx4 (&oh)[HAS_DELTA ? 1 : 4]) {
            const int rl = rl0 + X.c32 < nrows ? rl0 + X.c32 : nrows - 1;
            x.rvalid = rl0 + X.c32 < nrows;
            x.ri = (int)fdiv((unsigned)rl, a.div_g);
            const int gq = rl - x.ri * a.G;
            const long long qoff = (long long)x.ri * a.q_ss + (long long)gq * a.q_sh + 8 * X.h + 64 * DH;
            const long long ooff = (long long)x.ri * a.o_ss + (long long)gq * a.o_sh + 8 * X.h + 64 * DH;
            x.lse_row = a.lse[((long long)b * a.Hq + k * a.G + gq) * a.S + x.ri];
            x.drow = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x.qh[i] = ld_global16(qb + qoff + 16 * i);
                x.doh[i] = ld_global16(dob + ooff + 16 * i);
                if constexpr (!HAS_DELTA)
                    oh[i] = ld_global16(outb + ooff + 16 * i);
            }
            if constexpr (HAS_DELTA) // left there by the dq kernel (the clamped row is a valid one, hence written)
                x.drow = g.delta[delta_index(a, b, k * a.G + gq, x.ri)];
        };
        // The blocks that hold a row with i >= k0, from the candidate's last block down to the first
        // such one: the units of one (candidate, KV head) pair run side by side on one XCD (see the
        // kernel), and walking downwards they all ask for the same rows of q and dout at about the same
        // time, whatever their tile, so that those rows come from HBM once and from that XCD's L2 after.
        const int rl_first = (k0 * a.G) / kBlockRows * kBlockRows;
        const int rl_last = (nrows - 1) / kBlockRows * kBlockRows;
        // With <dout,out> at hand (no rows of out to fetch) there are registers to spare: the next
        // block is requested while the current one is worked on.
        constexpr bool kAhead = HAS_DELTA;
        BlockIn nx;
        uintx4 oh[HAS_DELTA ? 1 : 4];
        if constexpr (kAhead) {
            fetch(rl_last, nx, oh);
            __builtin_amdgcn_s_waitcnt(0x0F70); // nothing in flight at the loop's entry either (see its end)
        }
        for (int rl0 = rl_last; rl0 >= rl_first; rl0 -= kBlockRows) {
            BlockIn cur;
            if constexpr (kAhead) {
                cur = nx;
                if (rl0 - kBlockRows >= rl_first)
                    fetch(rl0 - kBlockRows, nx, oh);
            } else {
                fetch(rl0, cur, oh);
            }
            const uintx4 (&qh)[4] = cur.qh;
            const uintx4 (&doh)[4] = cur.doh;
            const bool rvalid = cur.rvalid;
            const int ri = cur.ri;
            const float lse_row = cur.lse_row * kLog2e;
            float drow = cur.drow;

            floatx16 s, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s[e] = 0.f;
                dp[e] = 0.f;
            }
            // dO^T and Q^T for the second products (independent of what follows: under the first products)
            bf16x8 at[2][2][2];
            transpose_halves(X, doh, qh, at);
            // this half of the two sums over the columns
#pragma unroll
            for (int i = 0; i < 4; ++i)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qh[i]), as_bf16x8(kfh[i]), s, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(doh[i]), as_bf16x8(vfh[i]), dp, 0, 0, 0);
            if constexpr (!HAS_DELTA) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        drow = __builtin_fmaf(bf16_lo(doh[i][e]), bf16_lo(oh[i][e]), drow);
                        drow = __builtin_fmaf(bf16_hi(doh[i][e]), bf16_hi(oh[i][e]), drow);
                    }
                drow += __shfl_xor(drow, 32, 64); // this wavefront's 64 columns
            }
            // The halves change hands.  Each wavefront completes S and dP for one of the block's two
            // 16-row steps only (wavefront DH: rows 16*DH .. 16*DH+15, accumulator elements 8*DH .. 8*DH+7):
            // it hands over its half of the other step's sums and later receives that step's finished
            // weights, so that the exponentials are taken once per element and not once per wavefront.
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const int e0 = 4 * (2 * (1 - DH) + i2); // elements of the other wavefront's step
                *(lds_f32x4 *)(xch_mine + i2 * 1024) = floatx4{s[e0], s[e0 + 1], s[e0 + 2], s[e0 + 3]};
                *(lds_f32x4 *)(xch_mine + 2048 + i2 * 1024) = floatx4{dp[e0], dp[e0 + 1], dp[e0 + 2], dp[e0 + 3]};
            }
            if constexpr (!HAS_DELTA)
                if (X.h == 0)
                    xdrow[DH * 32 + X.c32] = drow;
            __syncthreads();
            float sf[8], dpf[8];
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const int e0 = 4 * (2 * DH + i2);
                const floatx4 so = *(lds_f32x4 *)(xch_other + i2 * 1024), dpo = *(lds_f32x4 *)(xch_other + 2048 + i2 * 1024);
#pragma unroll
                for (int t2 = 0; t2 < 4; ++t2) {
                    // the halves are added in a fixed order (columns 0..63 first), whichever wavefront does it
                    sf[4 * i2 + t2] = DH == 0 ? s[e0 + t2] + so[t2] : so[t2] + s[e0 + t2];
                    dpf[4 * i2 + t2] = DH == 0 ? dp[e0 + t2] + dpo[t2] : dpo[t2] + dp[e0 + t2];
                }
            }
            if constexpr (!HAS_DELTA) {
                const float other = xdrow[(1 - DH) * 32 + X.c32];
                drow = DH == 0 ? drow + other : other + drow;
            }
            // row quantities to LDS, then each lane fetches those of the 8 rows its elements of this step belong to
            if (X.h == 0) {
                aux_lse[X.c32] = lse_row;
                aux_drow[X.c32] = drow;
                aux_i[X.c32] = rvalid ? (float)ri : -1.f;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            float p[8], ds[8];
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2) {
                const int kk = 2 * DH + i2;
                const floatx4 l4 = *(lds_f32x4 *)(aux_lse + 8 * kk + 4 * X.h);
                const floatx4 d4 = *(lds_f32x4 *)(aux_drow + 8 * kk + 4 * X.h);
                const floatx4 i4 = *(lds_f32x4 *)(aux_i + 8 * kk + 4 * X.h);
#pragma unroll
                for (int t2 = 0; t2 < 4; ++t2) {
                    const int e = 4 * i2 + t2;
                    // the row sees suffix key `key` iff key <= its position (and the key exists)
                    const bool vis = (float)key <= i4[t2] && key < len;
                    p[e] = vis ? fast_exp2(__builtin_fmaf(sf[e], X.c, -l4[t2])) : 0.f;
                    ds[e] = p[e] * (dpf[e] - d4[t2]);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // this step's packed weights and score gradients go to the other wavefront, the other step's come back
            uintx4 pfp_u[2], pfs_u[2];
            pfp_u[DH] = uintx4{pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
            pfs_u[DH] = uintx4{pack_bf16(ds[0], ds[1]), pack_bf16(ds[2], ds[3]), pack_bf16(ds[4], ds[5]), pack_bf16(ds[6], ds[7])};
            *(lds_u128 *)(xch_mine + 4096) = pfp_u[DH];
            *(lds_u128 *)(xch_mine + 4096 + 1024) = pfs_u[DH];
            __syncthreads(); // also: the other wavefront has read this block's sums before the next block's are written
            pfp_u[1 - DH] = *(lds_u128 *)(xch_other + 4096);
            pfs_u[1 - DH] = *(lds_u128 *)(xch_other + 4096 + 1024);
            const bf16x8 pfp[2] = {as_bf16x8(pfp_u[0]), as_bf16x8(pfp_u[1])}, pfs[2] = {as_bf16x8(pfs_u[0]), as_bf16x8(pfs_u[1])};
            // the second products: this half of the columns of dV^T and dK^T
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) {
                    dv[i2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[j][0][i2], pfp[j], dv[i2], 0, 0, 0);
                    dk[i2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[j][1][i2], pfs[j], dk[i2], 0, 0, 0);
                }
            // The requests for the next block have had the whole block's work to land; waiting for them
            // here, in so many words, keeps the compiler from waiting for them at the top of the loop,
            // before the matrix instructions that do not need them (its bookkeeping of loads in flight
            // across the loop's back edge is coarse).
            if constexpr (kAhead)
                __builtin_amdgcn_s_waitcnt(0x0F70); // vector memory counter at zero, the others untouched
            // (No barrier here: what this wavefront writes next for the other one - the next block's sums - is
            // read by it after the next barrier only, and it has read this block's before it reached the last one.)
        }
    }
    const bool kvalid = key < len;
    // where this lane's rows of the gradients go (worked out here, not before the loop: no registers held across it)
    unsigned short *dst_k[4], *dst_v[4];
    bool dst_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int jr = k0 + 8 * u + (X.lane >> 3);
        dst_ok[u] = jr < a.S;
        const long long off = (long long)b * a.ks_sb + (long long)(dst_ok[u] ? jr : 0) * a.ks_ss + (long long)k * a.ks_sh +
                              8 * (X.lane & 7);
        dst_k[u] = reinterpret_cast<unsigned short *>(g.dk) + off;
        dst_v[u] = reinterpret_cast<unsigned short *>(g.dv) + off;
    }
    // the store routine addresses accumulators by column group: hand it this half in its place
    const floatx16 dk4[4] = {dk[0], dk[1], dk[0], dk[1]}, dv4[4] = {dv[0], dv[1], dv[0], dv[1]};
    store_rows<DH, DH>(X, dst_k, dst_ok, kvalid, a.scale, dk4);
    store_rows<DH, DH>(X, dst_v, dst_ok, kvalid, 1.0f, dv4);
}

template <bool HAS_DELTA>
__global__ __attribute__((amdgpu_flat_work_group_size(kDkvWaves * 64, kDkvWaves * 64), amdgpu_waves_per_eu(2, 4)))
void bwd_dkv_mfma_kernel(BwdArgs g, int nkt)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    // One unit - (candidate, KV head, 32-key tile) - per workgroup, one half of the output columns per
    // wavefront.  Workgroup ids go round the XCDs: the tiles of one (candidate, KV head) pair take
    // consecutive ids on ONE of them, so that they run there at the same time and share its L2.
    const int x = blockIdx.x & 7, y = blockIdx.x >> 3;
    const int grp = y / nkt, kt = y - grp * nkt;
    const long long bk = (long long)grp * 8 + x;
    if (bk >= (long long)g.f.B * g.f.Hkv) // the pairs are padded to a multiple of 8 (the same for the whole workgroup)
        return;
    // (wave-uniform branch; both sides meet the same workgroup barriers the same number of times)
    if (__builtin_amdgcn_readfirstlane(tid >> 6))
        bwd_dkv_unit<1, HAS_DELTA>(g, smem, tid, (int)bk, kt);
    else
        bwd_dkv_unit<0, HAS_DELTA>(g, smem, tid, (int)bk, kt);
}

} // namespace

bool bwd_mfma_supported(const Args &a, int dtype)
{
    return mfma_supported(a, dtype);
}

hipError_t launch_bwd_dkv_mfma(const BwdArgs &g, hipStream_t stream)
{
    const Args &a = g.f;
    const int nkt = (a.S + kTileKeys - 1) / kTileKeys;
    const long long nunits = ((long long)a.B * a.Hkv + 7) / 8 * 8 * nkt; // one workgroup each; pairs padded to a multiple of 8
    if (nunits > 0x7fffffffLL)
        return hipErrorInvalidValue;
    if (g.delta)
        return launch_kernel(bwd_dkv_mfma_kernel<true>, dim3((unsigned)nunits), dim3(kDkvWaves * 64), kDkvLdsBytes, stream, g, nkt);
    else
        return launch_kernel(bwd_dkv_mfma_kernel<false>, dim3((unsigned)nunits), dim3(kDkvWaves * 64), kDkvLdsBytes, stream, g, nkt);
}

hipError_t noalloc_scratch(void **ptr)
{
    static std::mutex mu;
    static void *by_device[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= kMaxDevices)
        return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(mu);
    if (!by_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return e;
        if (!p)
            return hipErrorInvalidSymbol;
        by_device[dev] = p;
    }
    *ptr = by_device[dev];
    return hipSuccess;
}

hipError_t launch_bwd_dq_mfma(const BwdArgs &g, hipStream_t stream)
{
    static DeviceSlots cu_by_device;
    hipError_t e;
    const int num_cu = device_setup_once(cu_by_device, e, [] {
        hipError_t s = hipFuncSetAttribute(reinterpret_cast<const void *>(bwd_dq_mfma_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kBwdLdsBytes);
        if (s == hipSuccess)
            s = hipFuncSetAttribute(reinterpret_cast<const void *>(bwd_dq_resident_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    2 * kDqMaxTiles * kTileBytes + kNW * kScrBytes);
        return s;
    });
    if (num_cu == 0)
        return e;
    const Args &a = g.f;
    const long long rows = (long long)a.C * a.S * a.G;
    // Short prefixes stay resident in LDS (the split of the workgroups over the (instruction, KV
    // head) pairs is that of the resident forward kernel).
    if (a.P <= kDqMaxTiles * kTileKeys && rows % kBlockRows == 0 && ((long long)a.S * a.G) % kBlockRows == 0 &&
        block_offsets_fit(a)) {
        const int max_tiles = (a.P + kTileKeys - 1) / kTileKeys;
        const long long nblocks = rows / kBlockRows;
        const long long VH = (long long)a.Np * a.Hkv;
        const long long vh_slots = VH < num_cu ? VH : num_cu;
        long long per_vh = num_cu / vh_slots;
        const long long useful = (nblocks + kNW - 1) / kNW;
        if (per_vh > useful)
            per_vh = useful;
        const size_t lds = (size_t)2 * max_tiles * kTileBytes + kNW * kScrBytes;
        return launch_kernel(bwd_dq_resident_kernel, dim3((unsigned)(per_vh * vh_slots)), dim3(kNW * 64), lds, stream, g,
                           (int)per_vh, (int)vh_slots, max_tiles);
    }
    const long long npasses = ((rows + kBwdPassRows - 1) / kBwdPassRows) * a.Np * a.Hkv;
    // two workgroups fit a compute unit's LDS; registers allow one, so one per compute unit
    const unsigned grid = (unsigned)(npasses < num_cu ? npasses : num_cu);
    return launch_kernel(bwd_dq_mfma_kernel, dim3(grid), dim3(kNW * 64), kBwdLdsBytes, stream, g, (int)npasses);
}

} // namespace pskv
