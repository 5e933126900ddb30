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
// Two kernels share this layout.  The general one handles any shape.  The pipelined one
// handles the common case in which every 32-row block lies inside one candidate and the
// suffix fits one 32-key step: it overlaps, inside each wavefront, the score product of the
// next tile (matrix cores) with the exponentials of the current one (vector ALU), requests
// everything it needs from global memory a full block ahead, and never branches on data.
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

// ------------------------------------------------------------------------------------------
// Shared per-lane context
// ------------------------------------------------------------------------------------------
struct Ctx {
    int lane, h, c32, head, Mtot;
    float c;          // softmax scale in log2 units
    lds_u8 *k_lane;   // K images + lane*16
    lds_u8 *v_lane;   // V images + lane*8
    lds_u8 *scr;      // this wavefront's V scratch
    int sv_row_lo;    // suffix V staging: key of this lane within a 16-key step (+ 8*(fragment & 1))
    int sv_chunk_lo;  // ... and its 16-byte chunk (+ 4*(fragment >> 1))
    const unsigned short *ksg, *vsg; // suffix K/V of this KV head
};

// Row bookkeeping of one lane for one 32-row block.
struct Row {
    unsigned rb, ri; // candidate and suffix position of the lane's row
    int rh;          // query head
    int rlen;        // suffix length of that candidate as stored (not yet clamped)
    bool rin;        // the row exists (r < B*S*G)
};

__device__ inline int clamp_len(const Args &a, int len) { return len < 0 ? 0 : (len > a.S ? a.S : len); }

// Wave-uniform clamped suffix length of candidate b.  Read through the constant address space
// (suf_len is never written during the call), which makes it a scalar load that does not queue
// behind the vector loads in flight.
__device__ inline int len_uniform(const Args &a, int b)
{
    typedef const __attribute__((address_space(4))) int *const_int_ptr;
    if (!a.len)
        return a.S;
    return clamp_len(a, ((const_int_ptr)(unsigned long long)a.len)[__builtin_amdgcn_readfirstlane(b)]);
}

__device__ inline Row decode_row(const Args &a, const Ctx &X, int blk)
{
    Row x;
    const int r = blk * kBlockRows + X.c32;
    x.rin = r < X.Mtot;
    const unsigned rr = x.rin ? r : X.Mtot - 1;
    const unsigned tok = fdiv(rr, a.div_g), gq = rr - tok * a.G;
    x.rb = fdiv(tok, a.div_s);
    x.ri = tok - x.rb * a.S;
    x.rh = X.head * a.G + gq;
    x.rlen = a.len ? a.len[x.rb] : a.S;
    return x;
}

// Q fragments of a block: lane (row c32, half h) holds d = 16*ks + 8*h ..+7 for ks = 0..7.
// Padded rows are loaded as they are: a row's values only ever reach its own column of S^T
// and O^T, and padded rows are stored as zero.
__device__ inline void load_q(const Args &a, const Ctx &X, const Row &x, uintx4 (&dst)[8])
{
    const unsigned short *qrow = reinterpret_cast<const unsigned short *>(a.q) + (long long)x.rb * a.q_sb +
                                 (long long)x.ri * a.q_ss + (long long)x.rh * a.q_sh + 8 * X.h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        dst[ks] = ld_global16(qrow + 16 * ks);
}

// Suffix K fragments of step (candidate b, keys k0..k0+31) straight from global memory in
// A-operand layout.  Rows past kmax are never visible: their address is clamped to row kmax
// (and to row 0, candidate B-1, so that the loads stay in bounds even when there is no step).
__device__ inline void load_suffix_k(const Args &a, const Ctx &X, int b, int k0, int kmax, uintx4 (&kf)[8])
{
    const int bc = b < a.B ? b : a.B - 1;
    int krow = k0 + X.c32 < kmax ? k0 + X.c32 : kmax;
    krow = krow > 0 ? krow : 0;
    const unsigned short *kp = X.ksg + (long long)bc * a.ks_sb + (long long)krow * a.ks_ss + 8 * X.h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        kf[ks] = ld_global16(kp + 16 * ks);
}

// Suffix V rows of both 16-key steps in scratch-image order (clamped like K: a clamped row is
// finite data that only ever meets weight 0).
__device__ inline void load_suffix_v(const Args &a, const Ctx &X, int b, int k0, int kmax, uintx4 (&vf)[2][4])
{
    const int bc = b < a.B ? b : a.B - 1;
    const unsigned short *vb = X.vsg + (long long)bc * a.ks_sb;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int frag = 2 * it + X.h; // fragment (dt = frag >> 1, u = frag & 1)
            int key = k0 + 16 * j + 8 * (frag & 1) + X.sv_row_lo;
            key = key < kmax ? key : kmax;
            key = key > 0 ? key : 0;
            vf[j][it] = ld_global16(vb + (long long)key * a.ks_ss + (4 * (frag >> 1) + X.sv_chunk_lo) * 8);
        }
}

// O^T += V^T P^T for one 16-key step whose V rows are in registers: through the scratch tile.
__device__ inline void pv_from_scratch(const Ctx &X, const uintx4 (&vstep)[4], bf16x8 pfj, floatx16 (&o)[4])
{
#pragma unroll
    for (int it = 0; it < 4; ++it)
        *(lds_u128 *)(X.scr + it * 1024 + X.lane * 16) = vstep[it];
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

// Normalise and store one block (the division by the softmax denominator of Eq. 2); padded
// rows are stored as zero.  In the accumulators a lane holds scattered 4-element pieces of its
// row; stored like that, every memory request would carry 16 bytes.  So the block goes through
// the wavefront's scratch tile in two passes (output columns 0..63, then 64..127), written by
// the owners of the rows and read back so that 8 consecutive lanes store 128 contiguous bytes
// of one row.  Scratch layout: row*128 + ((chunk ^ row%8) * 16), chunk = 16 bytes.
__device__ inline void store_block(const Args &a, const Ctx &X, int r0, const Row &row, bool rvalid, float m, float l,
                                   const floatx16 (&o)[4])
{
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) uintx2 lds_u64;
    const float ltot = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / ltot;
    // rows this lane stores: 8*u + lane/8 for u = 0..3, 16 bytes at chunk lane%8 of each pass
    unsigned short *dst[4];
    bool dst_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = r0 + 8 * u + (X.lane >> 3);
        dst_ok[u] = r < X.Mtot;
        const unsigned rr = dst_ok[u] ? r : X.Mtot - 1;
        const unsigned tok = fdiv(rr, a.div_g), gq = rr - tok * a.G;
        const unsigned b = fdiv(tok, a.div_s), i = tok - b * a.S;
        dst[u] = reinterpret_cast<unsigned short *>(a.out) + (long long)b * a.o_sb + (long long)i * a.o_ss +
                 (long long)(X.head * a.G + gq) * a.o_sh + 8 * (X.lane & 7);
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int dt = 2 * pass + dl;
                uintx2 w = {0u, 0u};
                if (rvalid) { // a padded row may carry NaN; it is stored as zero
                    w[0] = pack_bf16(o[dt][4 * kk + 0] * inv, o[dt][4 * kk + 1] * inv);
                    w[1] = pack_bf16(o[dt][4 * kk + 2] * inv, o[dt][4 * kk + 3] * inv);
                }
                *(lds_u64 *)(X.scr + X.c32 * 128 + (((4 * dl + kk) ^ (X.c32 & 7)) << 4) + 8 * X.h) = w;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int rl = 8 * u + (X.lane >> 3);
            const uintx4 v = *(lds_u128 *)(X.scr + rl * 128 + (((X.lane & 7) ^ (rl & 7)) << 4));
            if (dst_ok[u])
                *reinterpret_cast<uintx4 *>(dst[u] + 64 * pass) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (row.rin && a.lse && X.h == 0)
        a.lse[((long long)row.rb * a.Hq + row.rh) * a.S + row.ri] =
            rvalid ? (m + __builtin_log2f(ltot)) * kLn2 : -INFINITY;
}

// Zeros for a block that holds nothing but padding.
__device__ inline void store_zero_block(const Args &a, const Ctx &X, const Row &row)
{
    if (!row.rin)
        return;
    unsigned short *orow = reinterpret_cast<unsigned short *>(a.out) + (long long)row.rb * a.o_sb +
                           (long long)row.ri * a.o_ss + (long long)row.rh * a.o_sh;
#pragma unroll
    for (int u = 0; u < 8; ++u)
        *reinterpret_cast<uintx4 *>(orow + 64 * X.h + 8 * u) = uintx4{0, 0, 0, 0};
    if (a.lse && X.h == 0)
        a.lse[((long long)row.rb * a.Hq + row.rh) * a.S + row.ri] = -INFINITY;
}

// Copies the prefix K/V of one head into the fragment-major LDS images (whole workgroup of 512
// threads).  Slot i of a tile image is bytes [i*16, i*16+16); which (key, chunk) goes there
// follows from the layouts described at the top of the file.  Rows past the prefix are zero.
// All global loads are issued before the first LDS write, so their latencies overlap.
__device__ inline void stage_prefix(const Args &a, int head, int ntiles, lds_u8 *kimg, lds_u8 *vimg, int tid)
{
    const unsigned short *kpg = reinterpret_cast<const unsigned short *>(a.kp) + (long long)head * a.kp_sh;
    const unsigned short *vpg = reinterpret_cast<const unsigned short *>(a.vp) + (long long)head * a.kp_sh;
    const int k_row = tid & 31, k_chunk = tid >> 5; // K: key-in-tile, 16-byte chunk of the row
    const int p5 = tid & 31, fr = tid >> 5;         // V: piece within a 512-byte fragment, fragment id
    const int v_row = 16 * ((fr >> 1) & 1) + 8 * (fr & 1) + 4 * ((p5 >> 4) & 1) + ((p5 >> 1) & 3);
    const int v_chunk = 4 * (fr >> 2) + 2 * ((p5 >> 3) & 1) + (p5 & 1);
    uintx4 kv[kMaxTiles], vv[kMaxTiles];
#pragma unroll
    for (int kt = 0; kt < kMaxTiles; ++kt) {
        // clamped, in-bounds addresses for every slot; what lies past the prefix is zeroed below
        const int kkey = kt * kTileKeys + k_row, vkey = kt * kTileKeys + v_row;
        const int kc = kkey < a.P ? kkey : (a.P > 0 ? a.P - 1 : 0), vc = vkey < a.P ? vkey : (a.P > 0 ? a.P - 1 : 0);
        if (kt < ntiles) {
            kv[kt] = ld_global16(kpg + (long long)kc * a.kp_sp + k_chunk * 8);
            vv[kt] = ld_global16(vpg + (long long)vc * a.kp_sp + v_chunk * 8);
        }
    }
#pragma unroll
    for (int kt = 0; kt < kMaxTiles; ++kt) {
        if (kt < ntiles) {
            const int kkey = kt * kTileKeys + k_row, vkey = kt * kTileKeys + v_row;
            *(lds_u128 *)(kimg + kt * kTileBytes + tid * 16) = kkey < a.P ? kv[kt] : uintx4{0, 0, 0, 0};
            *(lds_u128 *)(vimg + kt * kTileBytes + tid * 16) = vkey < a.P ? vv[kt] : uintx4{0, 0, 0, 0};
        }
    }
}

__device__ inline Ctx make_ctx(const Args &a, lds_u8 *smem, int ntiles, int tid, int head)
{
    Ctx X;
    X.lane = tid & 63;
    X.h = X.lane >> 5;
    X.c32 = X.lane & 31;
    X.head = head;
    X.Mtot = a.B * a.S * a.G;
    X.c = a.scale * kLog2e;
    X.k_lane = smem + X.lane * 16;
    X.v_lane = smem + ntiles * kTileBytes + X.lane * 8;
    X.scr = smem + 2 * ntiles * kTileBytes + __builtin_amdgcn_readfirstlane(tid >> 6) * kScrBytes;
    X.sv_row_lo = 4 * ((X.c32 >> 4) & 1) + ((X.c32 >> 1) & 3);
    X.sv_chunk_lo = 2 * ((X.c32 >> 3) & 1) + (X.c32 & 1);
    X.ksg = reinterpret_cast<const unsigned short *>(a.ks) + (long long)head * a.ks_sh;
    X.vsg = reinterpret_cast<const unsigned short *>(a.vs) + (long long)head * a.ks_sh;
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
        store_zero_block(a, X, row);
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

    // ---- prefix part: every row sees every prefix key ----
    for (int kt = 0; kt < ntiles; ++kt) {
        floatx16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = as_bf16x8(*(lds_u128 *)(X.k_lane + kt * kTileBytes + ks * 1024));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, as_bf16x8(q[ks]), s, 0, 0, 0);
        }
        const int nvalid = a.P - kt * kTileKeys;
        if (nvalid < kTileKeys) { // ragged last tile: keys past the prefix are not visible
            const int nv = nvalid - 4 * X.h; // element e holds key 8*(e/4) + e%4 + 4*h of the tile
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (8 * (e >> 2) + (e & 3) >= nv)
                    s[e] = -INFINITY;
        }
        bf16x8 pf[2];
        softmax_tile(s, st, X.c, pf);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_fragment(X.v_lane + kt * kTileBytes, dt, j),
                                                                   pf[j], st.o[dt], 0, 0, 0);
    }

    // ---- suffix part: (candidate, 32-key step) pairs, wave-uniform ----
    const int last_row = r0 + kBlockRows - 1 < X.Mtot ? r0 + kBlockRows - 1 : X.Mtot - 1;
    const int tok_first = fdiv(r0, a.div_g), tok_last = fdiv(last_row, a.div_g);
    const int b_last = fdiv(tok_last, a.div_s);
    for (int b = fdiv(tok_first, a.div_s); b <= b_last; ++b) {
        const int len = len_uniform(a, b);
        const int i_lo = tok_first - b * a.S > 0 ? tok_first - b * a.S : 0;
        const int i_hi = tok_last - b * a.S < a.S - 1 ? tok_last - b * a.S : a.S - 1;
        const int kmax = i_hi < len - 1 ? i_hi : len - 1; // last suffix key any row of this block sees
        if (i_lo >= len)
            continue;
        for (int k0 = 0; k0 <= kmax; k0 += kTileKeys) {
            uintx4 kf[8], vf[2][4];
            load_suffix_k(a, X, b, k0, kmax, kf);
            load_suffix_v(a, X, b, k0, kmax, vf);
            // the row sees keys 0..ri of its own candidate; element e holds key k0 + 8*(e/4) + e%4 + 4*h
            const int lim = ((int)row.rb == b ? (int)row.ri : -1) - k0 - 4 * X.h;
            floatx16 s;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), as_bf16x8(q[ks]), s, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s[e] = 8 * (e >> 2) + (e & 3) <= lim ? s[e] : -INFINITY;
            bf16x8 pf[2];
            softmax_tile(s, st, X.c, pf);
            pv_from_scratch(X, vf[0], pf[0], st.o);
            pv_from_scratch(X, vf[1], pf[1], st.o);
        }
    }
    store_block(a, X, r0, row, rvalid, st.m, st.l, st.o);
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void resident_general_kernel(Args a, int wgs_per_head, int ntiles)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int head = blockIdx.x % a.Hkv; // consecutive workgroup ids (one per XCD in turn) take consecutive heads
    const Ctx X = make_ctx(a, smem, ntiles, tid, head);
    stage_prefix(a, head, ntiles, smem, smem + ntiles * kTileBytes, tid);
    __syncthreads();
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int blk = (blockIdx.x / a.Hkv) * kNW + wave; blk < nblocks; blk += wgs_per_head * kNW)
        general_block(a, X, ntiles, blk);
}

// ------------------------------------------------------------------------------------------
// Pipelined path.  Preconditions (checked by the launcher): S*G is a multiple of 32, so a
// 32-row block lies inside one candidate; S <= 32, so the suffix is one 32-key step; and the
// prefix has at least two tiles.
//
// Softmax without per-tile maxima: the first prefix tile fixes the row's reference maximum;
// later tiles take exp2 relative to it whatever their own maximum is (a larger score just gives
// a weight above one, which fp32 sums and bf16 weights hold at full relative precision).  If a
// row's sum ends up at or above kBig, the wavefront goes over all its blocks once more with
// the general path after its main loop (rare; kept out of the main loop so that it costs it no
// registers).
// ------------------------------------------------------------------------------------------

// One step of the software pipeline.  On entry `s` holds the raw scores of the current tile;
// the step computes the scores of the next tile (from LDS image `k_next`, or from the suffix K
// fragments `skf` when NEXT_FROM_REGS), the weights of the current tile and its value product
// from LDS image `v_cur`.  The eight score MFMAs are interleaved one to one with the weights
// of two score elements each, and from the fifth on with the value MFMAs of the first 16 keys.
// FRESH: the output accumulators start from zero here.
template <bool FRESH, bool NEXT_FROM_REGS>
__device__ __attribute__((always_inline)) void pipe_step(lds_u8 *k_next, const uintx4 (&skf)[8], lds_u8 *v_cur,
                                                         const uintx4 (&q)[8], floatx16 &s, float c, float m,
                                                         float &l, floatx16 (&o)[4])
{
    floatx16 sn;
#pragma unroll
    for (int e = 0; e < 16; ++e)
        sn[e] = 0.f;
    uintx4 kfr[8];
    bf16x8 vfr[2][4];
    unsigned pk[8];
    bf16x8 pf0;
    float rs = 0.f;
    if (!NEXT_FROM_REGS) {
        kfr[0] = *(lds_u128 *)(k_next);
        kfr[1] = *(lds_u128 *)(k_next + 1024);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        // LDS reads for later steps: K two steps ahead, V(dt = ks%4, j = ks/4) four steps ahead
        if (!NEXT_FROM_REGS && ks + 2 < 8)
            kfr[ks + 2] = *(lds_u128 *)(k_next + (ks + 2) * 1024);
        vfr[ks >> 2][ks & 3] = v_fragment(v_cur, ks & 3, ks >> 2);
        // matrix cores
        sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(NEXT_FROM_REGS ? skf[ks] : kfr[ks]), as_bf16x8(q[ks]),
                                                     sn, 0, 0, 0);
        if (ks >= 4) {
            floatx16 acc = o[ks - 4];
            if (FRESH) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    acc[e] = 0.f;
            }
            o[ks - 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[0][ks - 4], pf0, acc, 0, 0, 0);
        }
        // vector ALU: weights of elements 2ks and 2ks+1 of the current tile
        const float p0 = fast_exp2(__builtin_fmaf(s[2 * ks], c, -m));
        const float p1 = fast_exp2(__builtin_fmaf(s[2 * ks + 1], c, -m));
        rs += p0;
        rs += p1;
        pk[ks] = pack_bf16(p0, p1);
        if (ks == 3)
            pf0 = as_bf16x8(uintx4{pk[0], pk[1], pk[2], pk[3]});
        // Keep the step together: the empty asm makes this step's vector results exist here,
        // and nothing may be moved across the barrier that follows it.
        asm volatile("" : "+v"(rs), "+v"(pk[ks]));
        __builtin_amdgcn_sched_barrier(0);
    }
    const bf16x8 pf1 = as_bf16x8(uintx4{pk[4], pk[5], pk[6], pk[7]});
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[1][dt], pf1, o[dt], 0, 0, 0);
    l += rs;
    s = sn;
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void resident_pipelined_kernel(Args a, int wgs_per_head, int ntiles)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    const int tid = threadIdx.x;
    const int head = blockIdx.x % a.Hkv; // consecutive workgroup ids (one per XCD in turn) take consecutive heads
    const Ctx X = make_ctx(a, smem, ntiles, tid, head);
    const int nblocks = (X.Mtot + kBlockRows - 1) / kBlockRows;
    const int blk_stride = wgs_per_head * kNW;
    const int rows_per_cand = a.S * a.G; // a multiple of 32

    // First key a block's rows can see and last suffix position its rows have, from its index:
    // block blk covers rows [32*blk, 32*blk+31] of candidate 32*blk / (S*G).
    // A block whose first row is already past its candidate's length holds nothing but padding.
    auto block_cand = [&](int blk) { return (int)fdiv(fdiv(blk * kBlockRows, a.div_g), a.div_s); };
    auto block_i_lo = [&](int blk) { return (int)fdiv(blk * kBlockRows, a.div_g) - block_cand(blk) * a.S; };
    // Advance to the next block of this wavefront that has a valid row; blocks of pure padding
    // on the way are stored as zeros here and now.
    auto skip_padding = [&](int blk) {
        while (blk < nblocks && block_i_lo(blk) >= len_uniform(a, block_cand(blk))) {
            store_zero_block(a, X, decode_row(a, X, blk));
            blk += blk_stride;
        }
        return blk;
    };

    // first block of this wavefront: request its row decode and Q before the prefix copy
    const int first_blk = (blockIdx.x / a.Hkv) * kNW + __builtin_amdgcn_readfirstlane(tid >> 6);
    bool any_bad = false;
    int blk = skip_padding(first_blk);
    Row nxt = decode_row(a, X, blk < nblocks ? blk : nblocks - 1);
    uintx4 q[8]; // this block's Q fragments until their last use, then the next block's
    load_q(a, X, nxt, q);

    stage_prefix(a, head, ntiles, smem, smem + ntiles * kTileBytes, tid);
    __syncthreads();

    while (blk < nblocks) {
        const int r0 = blk * kBlockRows;
        const Row row = nxt;
        const bool rvalid = row.rin && (int)row.ri < clamp_len(a, row.rlen);

        // the block's suffix step: candidate sb, keys 0..skmax
        const int sb = block_cand(blk);
        const int i_hi = (int)fdiv(r0 + kBlockRows - 1, a.div_g) - sb * a.S;
        const int len = len_uniform(a, sb);
        const int skmax = i_hi < len - 1 ? i_hi : len - 1;
        // Loads are retired in issue order, so what is needed last is requested first.
        uintx4 skf[8], svf[2][4];
        load_suffix_k(a, X, sb, 0, skmax, skf);

        // ---- first prefix tile: scores, reference maximum ----
        floatx16 s;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s[e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(lds_u128 *)(X.k_lane + ks * 1024)), as_bf16x8(q[ks]), s,
                                                        0, 0, 0);
        float m = s[0];
#pragma unroll
        for (int e = 1; e < 16; ++e)
            m = fmaxf(m, s[e]);
        m = fmaxf(m, __shfl_xor(m, 32, 64)) * X.c; // the other half-wave holds the other 16 keys
        float l = 0.f;
        floatx16 o[4];

        // ---- pipeline over the prefix tiles: scores of tile kt+1 under the weights of tile kt ----
        pipe_step<true, false>(X.k_lane + kTileBytes, skf, X.v_lane, q, s, X.c, m, l, o);
        for (int kt = 1; kt < ntiles - 1; ++kt)
            pipe_step<false, false>(X.k_lane + (kt + 1) * kTileBytes, skf, X.v_lane + kt * kTileBytes, q, s, X.c, m, l, o);
        if (a.P & (kTileKeys - 1)) { // ragged last prefix tile: keys past the prefix are not visible
            const int nv = a.P - (ntiles - 1) * kTileKeys - 4 * X.h;
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (8 * (e >> 2) + (e & 3) >= nv)
                    s[e] = -INFINITY;
        }
        load_suffix_v(a, X, sb, 0, skmax, svf); // one tile ahead of its use
        // ---- last prefix tile: the "next scores" are the suffix scores, from the K registers ----
        pipe_step<false, true>(X.k_lane, skf, X.v_lane + (ntiles - 1) * kTileBytes, q, s, X.c, m, l, o);

        // Q has been used for the last time: the next block's row decode and Q take its place.
        // (Requested unconditionally, for a clamped block index past the end: a load under a
        // branch would have to be waited for and copied at the join.)
        blk = skip_padding(blk + blk_stride);
        nxt = decode_row(a, X, blk < nblocks ? blk : nblocks - 1);
        load_q(a, X, nxt, q);

        // ---- suffix step: causal mask, weights, value product through the scratch tile ----
        {
            const int lim = (int)row.ri - 4 * X.h; // the row sees keys 0..ri; element e holds key 8*(e/4) + e%4 + 4*h
            unsigned pk[8];
            float rs = 0.f;
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float s0 = 8 * (e >> 2) + (e & 3) <= lim ? s[e] : -INFINITY;
                const float s1 = 8 * ((e + 1) >> 2) + ((e + 1) & 3) <= lim ? s[e + 1] : -INFINITY;
                const float p0 = fast_exp2(__builtin_fmaf(s0, X.c, -m));
                const float p1 = fast_exp2(__builtin_fmaf(s1, X.c, -m));
                rs += p0;
                rs += p1;
                pk[e >> 1] = pack_bf16(p0, p1);
            }
            l += rs;
            pv_from_scratch(X, svf[0], as_bf16x8(uintx4{pk[0], pk[1], pk[2], pk[3]}), o);
            pv_from_scratch(X, svf[1], as_bf16x8(uintx4{pk[4], pk[5], pk[6], pk[7]}), o);
        }

        any_bad |= __builtin_amdgcn_ballot_w64(rvalid && !(l < kBig)) != 0;
        store_block(a, X, r0, row, rvalid, m, l, o);
    }

    // Rare: some row met scores far above its first tile's maximum.  Whatever this wavefront
    // stored is replaced by the general path's result.
    if (any_bad)
        for (int b2 = first_blk; b2 < nblocks; b2 += blk_stride)
            general_block(a, X, ntiles, b2);
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
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_general_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_pipelined_kernel),
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
    const bool pipelined = ((long long)a.S * a.G) % kBlockRows == 0 && a.S <= kTileKeys && ntiles >= 2;
    if (pipelined)
        hipLaunchKernelGGL(resident_pipelined_kernel, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_head, ntiles);
    else
        hipLaunchKernelGGL(resident_general_kernel, dim3(grid), dim3(kNW * 64), lds, stream, a, (int)per_head, ntiles);
    return hipGetLastError();
}

} // namespace pskv
