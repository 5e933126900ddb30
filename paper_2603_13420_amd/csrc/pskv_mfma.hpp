// Device code shared by the matrix-core kernels of batched candidate-suffix attention for
// gfx950 (bf16 tensors, head dim 128): operand layouts, the per-row softmax state, suffix
// loads, the output store and the software-pipelined tile step.
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
// LDS images of a 32-key tile are stored "fragment-major": the 16 bytes (K) or 8 bytes (V)
// that lane l reads for a given fragment sit at fragment_base + l*16 (or l*8), so every
// fragment read is one contiguous, conflict-free wave access with an immediate offset and no
// address arithmetic.
//   K image: fragment ks (16 d) at ks*1024; lane (key = l%32, h) holds d = 16*ks + 8*h ..+7
//   V image: fragment (dt, j, u) at ((dt*2 + j)*2 + u)*512; lane l = 32*h + 16*w + t names
//            key 16*j + 8*u + 4*h + t/4, d = 32*dt + 16*w + 4*(t%4) ..+3; the transposing
//            read then hands lane l the 4 keys 16*j + 8*u + 4*h + 0..3 at d = 32*dt + l%32.
// With both images a 16-byte chunk (key, c) of the row-major global tile lands at
// image_base + tid*16 when thread tid of a 512-thread group fetches the right (key, c):
// see TileSlot below.
#pragma once
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

// a * b with the rule that zero times anything, infinities and NaN included, is zero
// (v_mul_legacy_f32).  Bound to the compiler's own intrinsic rather than written as an inline
// instruction: the operands are matrix-core results, and the wait states a vector instruction
// needs after the matrix instruction that produced its input are inserted by the compiler only
// for instructions it emits itself - an inline one too close to the last matrix instruction
// reads the accumulator before it is written.
extern "C" __device__ float pskv_fmul_legacy(float, float) __asm("llvm.amdgcn.fmul.legacy");
__device__ inline float mul_zero_wins(float a, float b) { return pskv_fmul_legacy(a, b); }

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
    int lane, h, c32, Mtot; // Mtot: stacked rows of one (instruction, KV head) pair = C*S*G
    // the (instruction, KV head) pair being worked on ("virtual head")
    int head;   // KV head
    int cand0;  // first candidate of the instruction
    int P;      // real prefix rows of the instruction
    const unsigned short *kpg, *vpg; // first real prefix row of this instruction and KV head
    float c;          // softmax scale in log2 units
    lds_u8 *k_lane;   // K images + lane*16
    lds_u8 *v_lane;   // V images + lane*8
    lds_u8 *scr;      // this wavefront's V scratch
    int sv_row_lo;    // suffix V staging: key of this lane within a 16-key step (+ 8*(fragment & 1))
    int sv_chunk_lo;  // ... and its 16-byte chunk (+ 4*(fragment >> 1))
    const unsigned short *ksg, *vsg; // suffix K/V of this KV head
};

// Points the context at virtual head vh = instruction * Hkv + KV head: the instruction's real
// prefix rows are the last plen[instruction] of its P padded rows (App. F.1: the prefix is
// left-padded), so its prefix simply starts that much later and is that much shorter.
__device__ inline void set_vhead(const Args &a, Ctx &X, int vh)
{
    typedef const __attribute__((address_space(4))) int *const_int_ptr;
    const int n = vh / a.Hkv;
    X.head = vh - n * a.Hkv;
    X.cand0 = n * a.C;
    int pl = a.P;
    if (a.plen) {
        pl = ((const_int_ptr)(unsigned long long)a.plen)[__builtin_amdgcn_readfirstlane(n)];
        pl = pl < 0 ? 0 : (pl > a.P ? a.P : pl);
    }
    X.P = pl;
    const long long off = (long long)n * a.kp_sn + (long long)(a.P - pl) * a.kp_sp + (long long)X.head * a.kp_sh;
    X.kpg = reinterpret_cast<const unsigned short *>(a.kp) + off;
    X.vpg = reinterpret_cast<const unsigned short *>(a.vp) + off;
    X.ksg = reinterpret_cast<const unsigned short *>(a.ks) + (long long)X.head * a.ks_sh;
    X.vsg = reinterpret_cast<const unsigned short *>(a.vs) + (long long)X.head * a.ks_sh;
}

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

__device__ inline Row decode_row(const Args &a, const Ctx &X, int blk, int head, int cand0)
{
    Row x;
    const int r = blk * kBlockRows + X.c32;
    x.rin = r < X.Mtot;
    const unsigned rr = x.rin ? r : X.Mtot - 1;
    const unsigned tok = fdiv(rr, a.div_g), gq = rr - tok * a.G;
    const unsigned bl = fdiv(tok, a.div_s); // candidate within the instruction
    x.rb = cand0 + bl;
    x.ri = tok - bl * a.S;
    x.rh = head * a.G + gq;
    x.rlen = a.len ? a.len[x.rb] : a.S;
    return x;
}

__device__ inline Row decode_row(const Args &a, const Ctx &X, int blk) { return decode_row(a, X, blk, X.head, X.cand0); }

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

// Stores a 32 x 128 block held as O^T accumulators (lane column = row of the block), scaled by
// inv and rounded to bf16; rows with rvalid false are stored as zero.  In the accumulators a
// lane holds scattered 4-element pieces of its row; stored like that, every memory request
// would carry 16 bytes.  So the block goes through the wavefront's scratch tile in two passes
// (output columns 0..63, then 64..127), written by the owners of the rows and read back so that
// 8 consecutive lanes store 128 contiguous bytes of one row.  This lane stores rows
// 8*u + lane/8 (u = 0..3): dst[u] points at column 8*(lane%8) of that row, dst_ok[u] says
// whether the row exists.  Scratch layout: row*128 + ((chunk ^ row%8) * 16), chunk = 16 bytes.
// FIRST_PASS, LAST_PASS: the passes to run (0..1: all 128 columns; p..p: only columns 64p..64p+63).
template <int FIRST_PASS = 0, int LAST_PASS = 1>
__device__ inline void store_rows(const Ctx &X, unsigned short *const (&dst)[4], const bool (&dst_ok)[4], bool rvalid,
                                  float inv, const floatx16 (&o)[4])
{
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) uintx2 lds_u64;
    const float scale = rvalid ? inv : 0.f;
#pragma unroll
    for (int pass = FIRST_PASS; pass <= LAST_PASS; ++pass) {
#pragma unroll
        for (int dl = 0; dl < 2; ++dl)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int dt = 2 * pass + dl;
                // a padded row may carry NaN or infinities; scaled by a zero that wins it is stored as zero
                const uintx2 w = {pack_bf16(mul_zero_wins(o[dt][4 * kk + 0], scale), mul_zero_wins(o[dt][4 * kk + 1], scale)),
                                  pack_bf16(mul_zero_wins(o[dt][4 * kk + 2], scale), mul_zero_wins(o[dt][4 * kk + 3], scale))};
                *(lds_u64 *)(X.scr + X.c32 * 128 + (((4 * dl + kk) ^ (X.c32 & 7)) << 4) + 8 * X.h) = w;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int rl = 8 * u + (X.lane >> 3);
            const uintx4 v = *(lds_u128 *)(X.scr + rl * 128 + (((X.lane & 7) ^ (rl & 7)) << 4));
            if (dst_ok[u])
                // written once and not read again here: streaming stores keep the result from
                // piling up in L2, where it would wait for the write-back at the kernel's end
                __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(dst[u] + 64 * pass));
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Normalise and store one block of the output (the division by the softmax denominator of
// Eq. 2); padded rows are stored as zero.
__device__ inline void store_block(const Args &a, const Ctx &X, int r0, const Row &row, bool rvalid, float m, float l,
                                   const floatx16 (&o)[4])
{
    const float ltot = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / ltot;
    unsigned short *dst[4];
    bool dst_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = r0 + 8 * u + (X.lane >> 3);
        dst_ok[u] = r < X.Mtot;
        const unsigned rr = dst_ok[u] ? r : X.Mtot - 1;
        const unsigned tok = fdiv(rr, a.div_g), gq = rr - tok * a.G;
        const unsigned bl = fdiv(tok, a.div_s), i = tok - bl * a.S;
        dst[u] = reinterpret_cast<unsigned short *>(a.out) + (long long)(X.cand0 + bl) * a.o_sb + (long long)i * a.o_ss +
                 (long long)(X.head * a.G + gq) * a.o_sh + 8 * (X.lane & 7);
    }
    store_rows(X, dst, dst_ok, rvalid, inv, o);
    if (row.rin && a.lse && X.h == 0)
        a.lse[((long long)row.rb * a.Hq + row.rh) * a.S + row.ri] =
            rvalid ? (m + __builtin_log2f(ltot)) * kLn2 : -INFINITY;
}

// Zeros for the block of rows r0..r0+31 of the instruction, which holds nothing but padding; row
// is this lane's own row of the block.  Stored like a computed block, 128 contiguous bytes of a
// row per 8 lanes and instruction (whole cache lines, not sixteenths of them).
__device__ inline void store_zero_block(const Args &a, const Ctx &X, int r0, const Row &row)
{
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = r0 + 8 * u + (X.lane >> 3);
        if (r < X.Mtot) {
            const unsigned tok = fdiv((unsigned)r, a.div_g), gq = r - tok * a.G;
            const unsigned bl = fdiv(tok, a.div_s), i = tok - bl * a.S;
            unsigned short *dst = reinterpret_cast<unsigned short *>(a.out) + (long long)(X.cand0 + bl) * a.o_sb +
                                  (long long)i * a.o_ss + (long long)(X.head * a.G + gq) * a.o_sh + 8 * (X.lane & 7);
            __builtin_nontemporal_store(uintx4{0, 0, 0, 0}, reinterpret_cast<uintx4 *>(dst));
            __builtin_nontemporal_store(uintx4{0, 0, 0, 0}, reinterpret_cast<uintx4 *>(dst + 64));
        }
    }
    if (row.rin && a.lse && X.h == 0)
        a.lse[((long long)row.rb * a.Hq + row.rh) * a.S + row.ri] = -INFINITY;
}

// ------------------------------------------------------------------------------------------
// Bookkeeping for a 32-row block that lies inside one candidate (S*G a multiple of 32).  The
// candidate is then the same for all lanes, so everything that depends on it - its length, its
// offset into q, out, lse and the suffix K/V - is scalar, and what is left per lane (position
// and head within the candidate) fits 32-bit byte offsets.  Precondition (launchers): one
// candidate's part of q, of out and of the suffix K/V spans less than 2^31 bytes.
// ------------------------------------------------------------------------------------------
struct BlockRows {
    int b;          // candidate (global index), wave-uniform
    int len;        // its clamped suffix length, wave-uniform
    int ri, rh;     // this lane's suffix position and query head
    unsigned q_off; // byte offset of the lane's row from the candidate's first q row
    unsigned o_off; // ... from the candidate's first out row
};

__device__ inline BlockRows decode_block(const Args &a, const Ctx &X, int blk, int head, int cand0)
{
    BlockRows x;
    const unsigned r0 = (unsigned)blk * kBlockRows;
    const int bl = __builtin_amdgcn_readfirstlane((int)fdiv(fdiv(r0, a.div_g), a.div_s)); // candidate within the instruction
    x.b = cand0 + bl;
    x.len = len_uniform(a, x.b);
    const unsigned r = r0 + X.c32;
    const unsigned tok = fdiv(r, a.div_g), gq = r - tok * a.G;
    x.ri = (int)tok - bl * a.S;
    x.rh = head * a.G + (int)gq;
    // Rows past the candidate's length take the query row of its last position instead of their
    // own: the padding (a sixth of the query tensor at the paper's length mix) is never fetched,
    // and what such rows compute is finite and stored as zero.
    const int rq = x.ri < x.len ? x.ri : (x.len > 0 ? x.len - 1 : 0);
    x.q_off = ((unsigned)rq * (unsigned)a.q_ss + (unsigned)x.rh * (unsigned)a.q_sh) * 2u;
    x.o_off = ((unsigned)x.ri * (unsigned)a.o_ss + (unsigned)x.rh * (unsigned)a.o_sh) * 2u;
    return x;
}

// Q fragments of the block (layout as in load_q).
__device__ inline void load_q_block(const Args &a, const Ctx &X, const BlockRows &x, uintx4 (&dst)[8])
{
    const unsigned char *base = reinterpret_cast<const unsigned char *>(a.q) + (long long)x.b * a.q_sb * 2;
    const unsigned char *qrow = base + (x.q_off + 16u * X.h);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        dst[ks] = *reinterpret_cast<const uintx4 *>(qrow + 32 * ks);
}

// Suffix K fragments and V rows of keys k0..k0+31 of the block's candidate (layouts and
// clamping as in load_suffix_k and load_suffix_v; kmax >= 0).
__device__ inline void load_suffix_k_block(const Args &a, const Ctx &X, int b, int k0, int kmax, uintx4 (&kf)[8])
{
    const unsigned char *base = reinterpret_cast<const unsigned char *>(X.ksg) + (long long)b * a.ks_sb * 2;
    const int krow = k0 + X.c32 < kmax ? k0 + X.c32 : kmax;
    const unsigned char *kp = base + ((unsigned)krow * (unsigned)a.ks_ss * 2u + 16u * X.h);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        kf[ks] = *reinterpret_cast<const uintx4 *>(kp + 32 * ks);
}

__device__ inline void load_suffix_v_block(const Args &a, const Ctx &X, int b, int k0, int kmax, uintx4 (&vf)[2][4])
{
    const unsigned char *base = reinterpret_cast<const unsigned char *>(X.vsg) + (long long)b * a.ks_sb * 2;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int frag = 2 * it + X.h; // fragment (dt = frag >> 1, u = frag & 1)
            int key = k0 + 16 * j + 8 * (frag & 1) + X.sv_row_lo;
            key = key < kmax ? key : kmax;
            vf[j][it] = *reinterpret_cast<const uintx4 *>(
                base + ((unsigned)key * (unsigned)a.ks_ss * 2u + (unsigned)(4 * (frag >> 1) + X.sv_chunk_lo) * 16u));
        }
}

// Normalise and store the block (as store_block).  Lane l stores rows 8*u + l/8 of the block,
// whose offsets it takes from the lanes that own those rows.
__device__ inline void store_block_rows(const Args &a, const Ctx &X, const BlockRows &x, float m, float l,
                                        const floatx16 (&o)[4])
{
    const float ltot = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / ltot;
    const bool rvalid = x.ri < x.len;
    unsigned char *base = reinterpret_cast<unsigned char *>(a.out) + (long long)x.b * a.o_sb * 2;
    unsigned short *dst[4];
    bool dst_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const unsigned off = (unsigned)__shfl((int)x.o_off, 8 * u + (X.lane >> 3), 64);
        dst[u] = reinterpret_cast<unsigned short *>(base + (off + 16u * (X.lane & 7)));
        dst_ok[u] = true;
    }
    store_rows(X, dst, dst_ok, rvalid, inv, o);
    if (a.lse && X.h == 0)
        a.lse[((long long)x.b * a.Hq + x.rh) * a.S + x.ri] = rvalid ? (m + __builtin_log2f(ltot)) * kLn2 : -INFINITY;
}

// Zeros for a block that holds nothing but padding (stored like a computed block: whole cache lines).
__device__ inline void store_zero_block_rows(const Args &a, const Ctx &X, const BlockRows &x)
{
    unsigned char *base = reinterpret_cast<unsigned char *>(a.out) + (long long)x.b * a.o_sb * 2;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const unsigned off = (unsigned)__shfl((int)x.o_off, 8 * u + (X.lane >> 3), 64);
        unsigned char *dst = base + (off + 16u * (X.lane & 7));
        __builtin_nontemporal_store(uintx4{0, 0, 0, 0}, reinterpret_cast<uintx4 *>(dst));
        __builtin_nontemporal_store(uintx4{0, 0, 0, 0}, reinterpret_cast<uintx4 *>(dst + 128));
    }
    if (a.lse && X.h == 0)
        a.lse[((long long)x.b * a.Hq + x.rh) * a.S + x.ri] = -INFINITY;
}

// Which 16-byte chunk of a row-major 32-key tile thread tid of a 512-thread group fetches so
// that, written at image_base + tid*16, the chunks form the fragment-major K and V images.
struct TileSlot {
    int k_row, k_chunk, v_row, v_chunk;
};

__device__ inline TileSlot make_tile_slot(int tid)
{
    TileSlot t;
    t.k_row = tid & 31;  // K: key within the tile ...
    t.k_chunk = tid >> 5; // ... and 16-byte chunk of its row
    const int p5 = tid & 31, fr = tid >> 5; // V: piece within a 512-byte fragment, fragment id
    t.v_row = 16 * ((fr >> 1) & 1) + 8 * (fr & 1) + 4 * ((p5 >> 4) & 1) + ((p5 >> 1) & 3);
    t.v_chunk = 4 * (fr >> 2) + 2 * ((p5 >> 3) & 1) + (p5 & 1);
    return t;
}

// This thread's K and V chunks of prefix tile kt (rows clamped into the prefix: what lies past
// it is zeroed when the chunks are written, see write_tile_chunks).
__device__ inline void load_tile_chunks(const Args &a, const Ctx &X, const TileSlot &t, int kt, uintx4 &kv, uintx4 &vv)
{
    const int last = X.P > 0 ? X.P - 1 : 0;
    const int kkey = kt * kTileKeys + t.k_row, vkey = kt * kTileKeys + t.v_row;
    kv = ld_global16(X.kpg + (long long)(kkey < X.P ? kkey : last) * a.kp_sp + t.k_chunk * 8);
    vv = ld_global16(X.vpg + (long long)(vkey < X.P ? vkey : last) * a.kp_sp + t.v_chunk * 8);
}

__device__ inline void write_tile_chunks(const Ctx &X, const TileSlot &t, int kt, lds_u8 *kimg, lds_u8 *vimg, int tid,
                                         const uintx4 &kv, const uintx4 &vv)
{
    const int kkey = kt * kTileKeys + t.k_row, vkey = kt * kTileKeys + t.v_row;
    *(lds_u128 *)(kimg + tid * 16) = kkey < X.P ? kv : uintx4{0, 0, 0, 0};
    *(lds_u128 *)(vimg + tid * 16) = vkey < X.P ? vv : uintx4{0, 0, 0, 0};
}

// Classic online-softmax step over one prefix tile whose images are in LDS (k_lane and v_lane
// already include the lane offsets lane*16 and lane*8); nvalid = prefix keys in this tile.
__device__ inline void prefix_tile_classic(const Ctx &X, lds_u8 *k_lane, lds_u8 *v_lane, int nvalid,
                                           const uintx4 (&q)[8], RowState &st)
{
    floatx16 s;
#pragma unroll
    for (int e = 0; e < 16; ++e)
        s[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = as_bf16x8(*(lds_u128 *)(k_lane + ks * 1024));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, as_bf16x8(q[ks]), s, 0, 0, 0);
    }
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
            st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_fragment(v_lane, dt, j), pf[j], st.o[dt], 0, 0, 0);
}

// Causal suffix part of one 32-row block in full generality: the block may span several
// candidates and a candidate's suffix several 32-key steps; (candidate, step) pairs are
// wave-uniform.
__device__ inline void suffix_classic(const Args &a, const Ctx &X, int r0, const Row &row, const uintx4 (&q)[8],
                                      RowState &st)
{
    const int last_row = r0 + kBlockRows - 1 < X.Mtot ? r0 + kBlockRows - 1 : X.Mtot - 1;
    const int tok_first = fdiv(r0, a.div_g), tok_last = fdiv(last_row, a.div_g);
    const int bl_last = fdiv(tok_last, a.div_s);
    for (int bl = fdiv(tok_first, a.div_s); bl <= bl_last; ++bl) { // candidates within the instruction
        const int b = X.cand0 + bl;
        const int len = len_uniform(a, b);
        const int i_lo = tok_first - bl * a.S > 0 ? tok_first - bl * a.S : 0;
        const int i_hi = tok_last - bl * a.S < a.S - 1 ? tok_last - bl * a.S : a.S - 1;
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
}

// Suffix step with a fixed reference maximum m (suffix steps after the first): raw scores s of the keys
// k0..k0+31 of the row's own candidate, causal mask, weights, value product through the
// scratch tile.
__device__ inline void suffix_step_fixed(const Ctx &X, int ri, int k0, const floatx16 &s, float m, float &l,
                                         const uintx4 (&svf)[2][4], floatx16 (&o)[4])
{
    const int lim = ri - k0 - 4 * X.h; // the row sees keys 0..ri; element e holds key k0 + 8*(e/4) + e%4 + 4*h
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

// ------------------------------------------------------------------------------------------
// Passes of the streamed forward kernels.
// ------------------------------------------------------------------------------------------
// A pass is one (virtual head, group of 256 stacked rows) pair; a virtual head is one
// (instruction, KV head) pair with its own prefix and its own C*S*G stacked rows.
//
// Pass ids are laid out for the L2 caches.  All (virtual head, group) pairs, head by head, form one
// list of items - the heads in the order 0, 8, 16, ..., 1, 9, 17, ..., so that neighbours in the
// list belong to different instructions of the multi-instruction form, whose prefixes differ in
// length, and every stretch of the list is a fair sample of them; the workgroups whose ids are x modulo 8 - one XCD, ids going round the XCDs -
// take pass ids p = 8*y + x, y = 0, 1, ..., 32 at a time, and what matters is which items those
// are.  (With items dealt out head by head, item = p, each XCD cycled through five heads of the
// 13B-shaped workload at once and one prefix request in eight went to memory.)
//   - Heads of fewer than 256 groups: XCD x takes the x-th eighth of the list, in order.  It
//     works on one head at a time and a head's prefix is fetched into one L2, two at a boundary.
//   - Longer heads: the list is cut into chunks of 32 items and XCD x takes the chunks x, x+8, ...
//     The whole chip then works on one head at a time, each XCD on its own 32 groups of it
//     (measured 4 % faster on the 13B-shaped workload than XCDs that own heads).
// Either way every XCD gets the same number of items to within one chunk; the ids past the end
// of the list hold nothing.
struct Pass {
    int vh, head, cand0; // virtual head = instruction * Hkv + KV head; first candidate of the instruction
    int blk;             // this wavefront's block (clamped to the last one)
    bool exists;         // the pass id holds an item (the same for the whole workgroup)
    bool active;         // ... and this wavefront's block exists
};

constexpr int kChunk = 32;           // items per chunk: the compute units of an XCD
constexpr int kLongHead = 8 * kChunk; // groups per head from which the chunked order is used

// Items per XCD in the first order, rounds times 32 in the second: pass ids = 8 * this.
__host__ __device__ inline long long pass_ids_per_xcd(long long items, long long ngroups)
{
    return ngroups < kLongHead ? (items + 7) / 8 : (items + 8 * kChunk - 1) / (8 * kChunk) * kChunk;
}

// (The launchers see to it that the pass ids, and with them the items, fit 31 bits.)
__device__ inline Pass make_pass(const Args &a, int p, int npasses, int nblocks, int wave)
{
    Pass ps;
    const int pc = p < npasses ? p : npasses - 1;
    const int VH = a.Np * a.Hkv;
    const int ngroups = (nblocks + kNW - 1) / kNW;
    const int items = VH * ngroups;
    const int x = pc & 7, y = pc >> 3;
    int item;
    bool in_list;
    if (ngroups < kLongHead) {
        const int per = (items + 7) >> 3;
        item = x * per + y;
        in_list = y < per && item < items;
    } else {
        item = ((y / kChunk) * 8 + x) * kChunk + y % kChunk;
        in_list = item < items;
    }
    ps.exists = p < npasses && in_list;
    item = in_list ? item : items - 1;
    const int hpos = item / ngroups; // place of the head in the list
    const int group = item - hpos * ngroups;
    {
        const int nfull = VH >> 3, rem = VH & 7; // residue r modulo 8 has nfull + (r < rem) heads
        const int cut = rem * (nfull + 1);
        const int r = hpos < cut ? hpos / (nfull + 1) : rem + (hpos - cut) / (nfull > 0 ? nfull : 1);
        const int k = hpos < cut ? hpos - r * (nfull + 1) : (hpos - cut) - (r - rem) * nfull;
        ps.vh = k * 8 + r;
    }
    const int n = ps.vh / a.Hkv;
    ps.head = ps.vh - n * a.Hkv;
    ps.cand0 = n * a.C;
    const int blk = group * kNW + wave;
    ps.active = ps.exists && blk < nblocks;
    ps.blk = blk < nblocks ? blk : nblocks - 1;
    return ps;
}

// Pass ids of the streamed kernels (see make_pass).
inline long long stream_pass_ids(const Args &a)
{
    const long long rows = (long long)a.C * a.S * a.G;
    const long long ngroups = ((rows + kBlockRows - 1) / kBlockRows + kNW - 1) / kNW;
    return 8 * pass_ids_per_xcd((long long)a.Np * a.Hkv * ngroups, ngroups);
}

// Fragments 0 and 1 of the images a pipeline step starts with, read during the step before.
constexpr int kDist = 2; // LDS fragments are read this many sub-steps before their use
struct Pre {
    uintx4 k[kDist];
    bf16x8 v[kDist];
};

// One tile step of the three-stage software pipeline.  With t the current tile, the step
//   - computes the raw scores of tile t+1 into sn     (HAS_QK; K fragments from LDS image k_next,
//                                                      or from the registers skf when FROM_REGS),
//   - turns the raw scores s of tile t into weights   (relative to the fixed reference m; MASK:
//     pc, packed bf16, and adds their sum to l         element e is visible iff its key offset
//                                                      8*(e/4) + e%4 is <= lim),
//   - adds tile t-1 to the output: O^T += V^T P^T     (HAS_PV; V image v_prev, weights pp;
//                                                      FRESH: the accumulators start from zero).
// Each of its eight sub-steps issues one score MFMA, one value MFMA and the vector work of two
// score elements, so that matrix cores and vector ALU stay evenly loaded throughout.  (The row
// sum uses plain additions: next to MFMA work the bf16 dot-product instruction costs several
// times more issue time than two additions.)  LDS fragments are read two sub-steps ahead; the first fragments of the images the following step starts with
// (k_after when NEXT_K, v_cur when NEXT_V) are read during sub-steps 6 and 7 into `pre`.
template <bool HAS_QK, bool FROM_REGS, bool HAS_PV, bool FRESH, bool MASK, bool NEXT_K, bool NEXT_V>
__device__ __attribute__((always_inline)) void pipe_tile(lds_u8 *k_next, const uintx4 (&skf)[8], lds_u8 *v_prev,
                                                         lds_u8 *k_after, lds_u8 *v_cur, Pre &pre,
                                                         const uintx4 (&q)[8], const floatx16 &s, floatx16 &sn, float c,
                                                         float m, int lim, float &l, const uintx4 (&pp)[2],
                                                         uintx4 (&pc)[2], floatx16 (&o)[4])
{
    uintx4 kfr[8];
    bf16x8 vfr[8];
    unsigned pk[8];
    float rs = 0.f;
    if (HAS_QK) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sn[e] = 0.f;
        if (!FROM_REGS) {
#pragma unroll
            for (int i = 0; i < kDist; ++i)
                kfr[i] = pre.k[i];
        }
    }
    if (HAS_PV) {
#pragma unroll
        for (int i = 0; i < kDist; ++i)
            vfr[i] = pre.v[i];
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        // LDS reads for later sub-steps and for the following step
        if (HAS_QK && !FROM_REGS && ks + kDist < 8)
            kfr[ks + kDist] = *(lds_u128 *)(k_next + (ks + kDist) * 1024);
        if (HAS_PV && ks + kDist < 8)
            vfr[ks + kDist] = v_fragment(v_prev, (ks + kDist) & 3, (ks + kDist) >> 2);
        if (NEXT_K && ks >= 8 - kDist)
            pre.k[ks - (8 - kDist)] = *(lds_u128 *)(k_after + (ks - (8 - kDist)) * 1024);
        if (NEXT_V && ks >= 8 - kDist)
            pre.v[ks - (8 - kDist)] = v_fragment(v_cur, ks - (8 - kDist), 0);
        // matrix cores
        if (HAS_QK)
            sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(FROM_REGS ? skf[ks] : kfr[ks]), as_bf16x8(q[ks]), sn, 0,
                                                         0, 0);
        if (HAS_PV) {
            floatx16 acc = o[ks & 3];
            if (FRESH && ks < 4) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    acc[e] = 0.f;
            }
            o[ks & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[ks], as_bf16x8(pp[ks >> 2]), acc, 0, 0, 0);
        }
        // vector ALU: weights of elements 2ks and 2ks+1 of the current tile
        float s0 = s[2 * ks], s1 = s[2 * ks + 1];
        if (MASK) {
            s0 = 8 * ((2 * ks) >> 2) + ((2 * ks) & 3) <= lim ? s0 : -INFINITY;
            s1 = 8 * ((2 * ks + 1) >> 2) + ((2 * ks + 1) & 3) <= lim ? s1 : -INFINITY;
        }
        const float p0 = fast_exp2(__builtin_fmaf(s0, c, -m));
        const float p1 = fast_exp2(__builtin_fmaf(s1, c, -m));
        pk[ks] = pack_bf16(p0, p1);
        rs += p0;
        rs += p1;
        // Keep the sub-step together: the empty asm makes its vector results exist here, and
        // nothing may be moved across the barrier that follows it.
        asm volatile("" : "+v"(rs), "+v"(pk[ks]));
        __builtin_amdgcn_sched_barrier(0);
    }
    l += rs;
    pc[0] = uintx4{pk[0], pk[1], pk[2], pk[3]};
    pc[1] = uintx4{pk[4], pk[5], pk[6], pk[7]};
}

} // namespace
} // namespace pskv
