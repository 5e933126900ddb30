// Resident-prefix MFMA kernel of batched candidate-suffix attention for gfx950
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
// Matrix-core formulation (v_mfma_f32_32x32x16_bf16, fp32 accumulate), transposed so that a
// lane owns one query column q = lane % 32:
//     S^T[key][q] = sum_d K[key][d] Q[q][d]           A = K fragment,  B = Q fragment
//     O^T[d][q]  += sum_key V[key][d] P^T[key][q]     A = V^T fragment, B = P^T fragment
// The accumulator of the first product holds, for lane half h = lane/32, keys 8*kk + 4*h + t
// of the tile in element 4*kk + t.  Elements 8j..8j+7 are used unchanged as the B fragment of
// contraction step j of the second product, which fixes the order in which V rows enter its
// A fragment: slot (h, e) of step j is key 16*j + 8*(e/4) + 4*h + e%4.
//
// LDS images are stored "fragment-major": the 16 bytes (K) or 8 bytes (V) that lane l reads
// for a given fragment sit at fragment_base + l*16 (or l*8), so every fragment read is one
// contiguous, conflict-free wave access with an immediate offset and no address arithmetic.
//   K tile (32 keys): fragment ks (16 d) at ks*1024; lane (key = l%32, h) holds d = 16*ks + 8*h ..+7
//   V tile (32 keys): fragment (dt, j, u) at ((dt*2 + j)*2 + u)*512; lane l = 32*h + 16*w + t names
//                     key 16*j + 8*u + 4*h + t/4, d = 32*dt + 16*w + 4*(t%4) ..+3; the transposing
//                     read then hands lane l the 4 keys 16*j + 8*u + 4*h + 0..3 at d = 32*dt + l%32.
// With both images a 16-byte chunk (key, c) of the row-major global tile lands at
// tile_base + tid*16 when thread tid of a 512-thread group fetches the right (key, c).
#include "pskv_internal.h"

namespace pskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kBlockRows = 32;          // query rows per wavefront block
constexpr int kNW = 8;                  // wavefronts per workgroup
constexpr int kTileKeys = 32;           // keys per LDS tile
constexpr int kTileBytes = kTileKeys * kD * 2; // 8 KB
constexpr int kMaxTiles = 8;            // resident prefix: at most 256 keys
constexpr int kScrBytes = 4096;         // per-wave V scratch: 16 keys
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kBig = 1.0e18f;         // row sums at or above this trigger a rescale

typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) uintx4 lds_u128;

__device__ inline unsigned fdiv(unsigned n, FastDiv d) { return (unsigned)(((unsigned long long)n * d.mul) >> d.shift); }

__device__ inline uintx4 ld_global16(const unsigned short *p) { return *reinterpret_cast<const uintx4 *>(p); }

__device__ inline bf16x8 as_bf16x8(uintx4 v)
{
    bf16x8 r;
    __builtin_memcpy(&r, &v, 16);
    return r;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ inline unsigned pack_bf16(float lo, float hi)
{
    floatx2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    unsigned r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

__device__ inline short4v lds_read_tr(lds_u8 *p)
{
    typedef short4v __attribute__((address_space(3))) * tr_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)p);
}

// A fragment of V^T for contraction step j of tile image `vt`, output-column tile dt.
__device__ inline bf16x8 v_fragment(lds_u8 *vt_lane, int dt, int j)
{
    short4v lo = lds_read_tr(vt_lane + ((dt * 2 + j) * 2 + 0) * 512);
    short4v hi = lds_read_tr(vt_lane + ((dt * 2 + j) * 2 + 1) * 512);
    short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    bf16x8 vf;
    __builtin_memcpy(&vf, &v8, 16);
    return vf;
}

struct RowState {
    float m;       // reference maximum of the scaled scores, log2 units (-inf: nothing seen yet)
    float l;       // this lane's share of the running sum (the other half-wave holds the rest)
    floatx16 o[4]; // O^T accumulators: o[dt][4*kk + t] = O^T[32*dt + 8*kk + 4*h + t][q]
};

// Softmax step for one 32-key tile whose raw (masked: -inf) scores are in s.
// Fast path: weights are taken relative to the row's current reference maximum without looking
// at this tile's maximum; exp2 of a larger score simply gives a weight above one, which fp32
// sums and bf16 weights hold at full relative precision.  Only when some row's tile sum is not
// below kBig (first tile of a row, or scores far above the reference) does the wavefront take
// the classic online-softmax step: new maximum, rescale of sum and output, weights recomputed.
__device__ inline void softmax_tile(const floatx16 &s, RowState &st, float c, bf16x8 (&pf)[2])
{
    float p[16];
    float rs = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        p[e] = fast_exp2(__builtin_fmaf(s[e], c, -st.m));
        rs += p[e];
    }
    if (__builtin_amdgcn_ballot_w64(!(rs < kBig)) != 0) {
        float tmax = s[0];
#pragma unroll
        for (int e = 1; e < 16; ++e)
            tmax = fmaxf(tmax, s[e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(st.m, tmax * c);
        const float msafe = mnew == -INFINITY ? 0.f : mnew; // nothing visible yet: weights all 0
        const float alpha = fast_exp2(st.m - msafe);
        st.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            st.o[dt] *= alpha;
        st.m = mnew;
        rs = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            p[e] = fast_exp2(__builtin_fmaf(s[e], c, -msafe));
            rs += p[e];
        }
    }
    st.l += rs;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        uintx4 w = {pack_bf16(p[8 * j + 0], p[8 * j + 1]), pack_bf16(p[8 * j + 2], p[8 * j + 3]),
                    pack_bf16(p[8 * j + 4], p[8 * j + 5]), pack_bf16(p[8 * j + 6], p[8 * j + 7])};
        pf[j] = as_bf16x8(w);
    }
}

// ALIGNED1: every 32-row block lies inside one candidate (S*G is a multiple of 32) and the
// suffix fits one 32-key step (S <= 32).
template <bool ALIGNED1>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void resident_kernel(Args a, int wgs_per_head, int ntiles)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    lds_u8 *kimg = smem;                       // [ntiles][8 KB]
    lds_u8 *vimg = smem + ntiles * kTileBytes; // [ntiles][8 KB]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, c32 = lane & 31;
    lds_u8 *scr = smem + 2 * ntiles * kTileBytes + wave * kScrBytes;

    const int head = blockIdx.x % a.Hkv; // consecutive workgroup ids (one per XCD in turn) take consecutive heads
    const int wg_in_head = blockIdx.x / a.Hkv;
    const int Mtot = a.B * a.S * a.G;
    const int nblocks = (Mtot + kBlockRows - 1) / kBlockRows;
    const float c = a.scale * kLog2e;

    const unsigned short *qg = reinterpret_cast<const unsigned short *>(a.q);
    const unsigned short *ksg = reinterpret_cast<const unsigned short *>(a.ks) + (long long)head * a.ks_sh;
    const unsigned short *vsg = reinterpret_cast<const unsigned short *>(a.vs) + (long long)head * a.ks_sh;
    const unsigned short *kpg = reinterpret_cast<const unsigned short *>(a.kp) + (long long)head * a.kp_sh;
    const unsigned short *vpg = reinterpret_cast<const unsigned short *>(a.vp) + (long long)head * a.kp_sh;
    unsigned short *og = reinterpret_cast<unsigned short *>(a.out);

    // ---- prefix K/V of this head -> LDS, once.  Thread tid fills bytes [tid*16, tid*16+16) of
    //      each tile image; which (key, chunk) that is follows from the fragment-major layouts.
    {
        const int k_row = tid & 31, k_chunk = tid >> 5; // K: key-in-tile, 16-byte chunk of the row
        const int p5 = tid & 31, blk = tid >> 5;        // V: piece within a 512-byte fragment, fragment id
        const int v_row = 16 * ((blk >> 1) & 1) + 8 * (blk & 1) + 4 * ((p5 >> 4) & 1) + ((p5 >> 1) & 3);
        const int v_chunk = 4 * (blk >> 2) + 2 * ((p5 >> 3) & 1) + (p5 & 1);
        for (int kt = 0; kt < ntiles; ++kt) {
            const int kkey = kt * kTileKeys + k_row, vkey = kt * kTileKeys + v_row;
            uintx4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0}; // rows past the prefix stay zero
            if (kkey < a.P)
                kv = ld_global16(kpg + (long long)kkey * a.kp_sp + k_chunk * 8);
            if (vkey < a.P)
                vv = ld_global16(vpg + (long long)vkey * a.kp_sp + v_chunk * 8);
            *(lds_u128 *)(kimg + kt * kTileBytes + tid * 16) = kv;
            *(lds_u128 *)(vimg + kt * kTileBytes + tid * 16) = vv;
        }
    }
    __syncthreads();

    lds_u8 *k_lane = kimg + lane * 16;
    lds_u8 *v_lane = vimg + lane * 8;
    lds_u8 *scr_lane = scr + lane * 8;

    // suffix V staging map for one 16-key step: iteration it covers fragments 2*it and 2*it+1
    const int sp5 = lane & 31;
    const int sv_row_lo = 4 * ((sp5 >> 4) & 1) + ((sp5 >> 1) & 3); // + 8*(fragment & 1)
    const int sv_chunk_lo = 2 * ((sp5 >> 3) & 1) + (sp5 & 1);     // + 4*(fragment >> 1)

    // Row bookkeeping of this lane for one block: candidate, suffix position, query head, and
    // the (still unclamped) suffix length of that candidate.
    struct Row {
        unsigned rb, ri;
        int rh, rlen;
        bool rin;
    };
    auto decode = [&](int blk) {
        Row x;
        const int r = blk * kBlockRows + c32;
        x.rin = r < Mtot;
        const unsigned rr = x.rin ? r : Mtot - 1;
        const unsigned tok = fdiv(rr, a.div_g), gq = rr - tok * a.G;
        x.rb = fdiv(tok, a.div_s);
        x.ri = tok - x.rb * a.S;
        x.rh = head * a.G + gq;
        x.rlen = a.len ? a.len[x.rb] : a.S;
        return x;
    };
    // Q fragments of a block: lane (row c32, half h) holds d = 16*ks + 8*h ..+7 for ks = 0..7.
    auto load_q = [&](const Row &x, uintx4 (&dst)[8]) {
        const unsigned short *qrow =
            qg + (long long)x.rb * a.q_sb + (long long)x.ri * a.q_ss + (long long)x.rh * a.q_sh + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            dst[ks] = ld_global16(qrow + 16 * ks);
    };
    // Wave-uniform clamped suffix length of candidate b (scalar load: it does not queue behind
    // the vector loads in flight).
    // (Read through the constant address space: suf_len is never written during the call.)
    typedef const __attribute__((address_space(4))) int *const_int_ptr;
    const const_int_ptr len_c = (const_int_ptr)(unsigned long long)a.len;
    auto len_of = [&](int b) {
        int len = a.len ? len_c[__builtin_amdgcn_readfirstlane(b)] : a.S;
        return len < 0 ? 0 : (len > a.S ? a.S : len);
    };

    const int blk_stride = wgs_per_head * kNW;
    int blk = wg_in_head * kNW + wave;
    Row nxt{};
    uintx4 qraw[8];
    if (blk < nblocks) {
        nxt = decode(blk);
        load_q(nxt, qraw);
    }

    while (blk < nblocks) {
        const int r0 = blk * kBlockRows;
        const int next_blk = blk + blk_stride;
        const Row cur = nxt;
        const int rlen = cur.rlen < 0 ? 0 : (cur.rlen > a.S ? a.S : cur.rlen);
        const bool rvalid = cur.rin && (int)cur.ri < rlen;
        const bool any_valid = __builtin_amdgcn_ballot_w64(rvalid) != 0; // else: nothing but padding
        unsigned short *orow =
            og + (long long)cur.rb * a.o_sb + (long long)cur.ri * a.o_ss + (long long)cur.rh * a.o_sh;
        // qraw holds this block's Q fragments until their last use, then the next block's.
        // Padded rows are used as they are: a row's values only ever reach its own column of
        // S^T and O^T, and padded rows are stored as zero.

        // ---- suffix steps of this block: (candidate, 32-key tile) pairs, wave-uniform ----
        const int last_row = r0 + kBlockRows - 1 < Mtot ? r0 + kBlockRows - 1 : Mtot - 1;
        const int tok_first = fdiv(r0, a.div_g), tok_last = fdiv(last_row, a.div_g);
        const int b_last = fdiv(tok_last, a.div_s);
        int sb = fdiv(tok_first, a.div_s), sk0 = 0, skmax = -1; // current step: candidate, first key, last key
        // advance (sb, sk0) to the next step that has a visible key; false when there is none
        auto seek = [&]() {
            while (sb <= b_last) {
                const int len = len_of(sb);
                const int i_lo = tok_first - sb * a.S > 0 ? tok_first - sb * a.S : 0;
                const int i_hi = tok_last - sb * a.S < a.S - 1 ? tok_last - sb * a.S : a.S - 1;
                skmax = i_hi < len - 1 ? i_hi : len - 1; // last suffix key any row of this block sees
                if (i_lo < len && sk0 <= skmax)
                    return true;
                ++sb;
                sk0 = 0;
            }
            return false;
        };
        // Suffix K fragments straight from global memory in A-operand layout.  Rows past skmax
        // are never visible: their address is clamped to row skmax instead of being zero-filled.
        uintx4 skf[8], svf[2][4];
        auto load_suffix_k = [&]() {
            const int bc = sb < a.B ? sb : a.B - 1; // when there is no step the loads still happen, in bounds
            int krow = sk0 + c32 < skmax ? sk0 + c32 : skmax;
            krow = krow > 0 ? krow : 0;
            const unsigned short *kp = ksg + (long long)bc * a.ks_sb + (long long)krow * a.ks_ss + 8 * h;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                skf[ks] = ld_global16(kp + 16 * ks);
        };
        // V rows of both 16-key steps in scratch-image order (clamped like K: a clamped row is
        // finite data that only ever meets weight 0)
        auto load_suffix_v = [&]() {
            const int bc = sb < a.B ? sb : a.B - 1;
            const unsigned short *vb = vsg + (long long)bc * a.ks_sb;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int frag = 2 * it + h; // fragment (dt = frag >> 1, u = frag & 1)
                    int key = sk0 + 16 * j + 8 * (frag & 1) + sv_row_lo;
                    key = key < skmax ? key : skmax;
                    key = key > 0 ? key : 0;
                    svf[j][it] = ld_global16(vb + (long long)key * a.ks_ss + (4 * (frag >> 1) + sv_chunk_lo) * 8);
                }
        };
        bool have_suf = any_valid && seek();
        load_suffix_k(); // needed last, requested first: loads retire in issue order

        RowState st;
        st.m = -INFINITY;
        st.l = 0.f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                st.o[dt][e] = 0.f;

        // ---- prefix part: every row sees every prefix key ----
        auto prefix_tile = [&](int kt) {
            floatx16 s;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 kf = as_bf16x8(*(lds_u128 *)(k_lane + kt * kTileBytes + ks * 1024));
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, as_bf16x8(qraw[ks]), s, 0, 0, 0);
            }
            const int nvalid = a.P - kt * kTileKeys;
            if (nvalid < kTileKeys) { // ragged last tile: keys past the prefix are not visible
                const int nv = nvalid - 4 * h; // element e holds key 8*(e/4) + e%4 + 4*h of the tile
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (8 * (e >> 2) + (e & 3) >= nv)
                        s[e] = -INFINITY;
            }
            bf16x8 pf[2];
            softmax_tile(s, st, c, pf);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_fragment(v_lane + kt * kTileBytes, dt, j),
                                                                       pf[j], st.o[dt], 0, 0, 0);
        };
        const int nt = any_valid ? ntiles : 0;
        for (int kt = 0; kt < nt - 1; ++kt)
            prefix_tile(kt);
        load_suffix_v(); // one tile ahead of its use
        if (nt > 0)
            prefix_tile(nt - 1);

        // ---- suffix part: causal attention to the own candidate's suffix K/V ----
        // One step (32 keys): scores, then - once the scores are out - `after_scores`, then
        // mask, softmax and the value product through the scratch tile.
        auto suffix_step = [&](auto after_scores) {
            // this row sees keys 0..ri of its own candidate; element e holds key sk0 + 8*(e/4) + e%4 + 4*h
            const int lim = ((int)cur.rb == sb ? (int)cur.ri : -1) - sk0 - 4 * h;
            floatx16 s;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(skf[ks]), as_bf16x8(qraw[ks]), s, 0, 0, 0);
            after_scores();
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s[e] = 8 * (e >> 2) + (e & 3) <= lim ? s[e] : -INFINITY;
            bf16x8 pf[2];
            softmax_tile(s, st, c, pf);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int it = 0; it < 4; ++it)
                    *(lds_u128 *)(scr + it * 1024 + lane * 16) = svf[j][it];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                bf16x8 va[4];
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    short4v lo = lds_read_tr(scr_lane + (dt * 2 + 0) * 512);
                    short4v hi = lds_read_tr(scr_lane + (dt * 2 + 1) * 512);
                    short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    __builtin_memcpy(&va[dt], &v8, 16);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt], pf[j], st.o[dt], 0, 0, 0);
            }
        };
        // The next block's row decode and Q go into the registers of this block's Q as soon as
        // those have been used for the last time.
        // (Requested unconditionally, for a clamped block index past the end: a load under a
        // branch would have to be waited for and copied at the join.)
        auto prefetch_next = [&]() {
            blk = next_blk;
            nxt = decode(blk < nblocks ? blk : nblocks - 1);
            load_q(nxt, qraw);
        };
        if (ALIGNED1) {
            // a block lies inside one candidate and the suffix fits one step: Q's last use is
            // that step's score product, everything after it runs under the prefetch
            if (have_suf)
                suffix_step(prefetch_next);
            else
                prefetch_next();
        } else {
            while (have_suf) {
                suffix_step([] {});
                sk0 += kTileKeys;
                have_suf = seek();
                if (have_suf) { // further steps (long suffixes, several candidates per block)
                    load_suffix_k();
                    load_suffix_v();
                }
            }
            prefetch_next();
        }

        // ---- normalise and store (the division by the softmax denominator of Eq. 2) ----
        const float ltot = st.l + __shfl_xor(st.l, 32, 64);
        if (cur.rin) {
            const float inv = rvalid ? 1.0f / ltot : 0.f;
            typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    uintx2 w = {0u, 0u};
                    if (rvalid) { // padded rows are stored as zero
                        w[0] = pack_bf16(st.o[dt][4 * kk + 0] * inv, st.o[dt][4 * kk + 1] * inv);
                        w[1] = pack_bf16(st.o[dt][4 * kk + 2] * inv, st.o[dt][4 * kk + 3] * inv);
                    }
                    *reinterpret_cast<uintx2 *>(orow + 32 * dt + 8 * kk + 4 * h) = w;
                }
            if (a.lse && h == 0)
                a.lse[((long long)cur.rb * a.Hq + cur.rh) * a.S + cur.ri] =
                    rvalid ? (st.m + __builtin_log2f(ltot)) * kLn2 : -INFINITY;
        }
    }
}

} // namespace

bool resident_supported(const Args &a)
{
    return a.D == kD && a.P <= kMaxTiles * kTileKeys;
}

hipError_t launch_resident(const Args &a, hipStream_t stream)
{
    static int num_cu = 0;
    if (num_cu == 0) {
        int dev = 0, n = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess)
            e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        const int max_lds = 2 * kMaxTiles * kTileBytes + kNW * kScrBytes;
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (e != hipSuccess)
            return e;
        num_cu = n > 0 ? n : 256;
    }
    const int ntiles = (a.P + kTileKeys - 1) / kTileKeys;
    const long long rows = (long long)a.B * a.S * a.G;
    const long long nblocks = (rows + kBlockRows - 1) / kBlockRows;
    // one workgroup per compute unit, split evenly over the KV heads; never more workgroups
    // per head than there are groups of 8 row blocks
    long long per_head = num_cu / a.Hkv > 0 ? num_cu / a.Hkv : 1;
    const long long useful = (nblocks + kNW - 1) / kNW;
    if (per_head > useful)
        per_head = useful;
    const unsigned grid = (unsigned)(per_head * a.Hkv);
    const size_t lds = (size_t)2 * ntiles * kTileBytes + kNW * kScrBytes;
    const bool aligned1 = ((long long)a.S * a.G) % kBlockRows == 0 && a.S <= kTileKeys;
    if (aligned1)
        hipLaunchKernelGGL(resident_kernel<true>, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_head, ntiles);
    else
        hipLaunchKernelGGL(resident_kernel<false>, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_head, ntiles);
    return hipGetLastError();
}

} // namespace pskv
