// MFMA path of batched candidate-suffix attention for gfx950 (bf16 tensors, head dim 128).
//
// All B*S suffix queries of one KV head (times the G query heads that share it) are stacked
// into one dense row dimension r = (b*S + i)*G + g  (suffix-centric alignment, Sec. 4.3: every
// suffix starts at column 0, so the stacking is a pure index map).  A workgroup owns 256
// consecutive rows and one KV head; each of its 8 wavefronts owns 32 rows.
//
// Prefix part (the 2*N_p term of App. B.1): the single shared prefix K/V is streamed through
// LDS in 64-key tiles, each tile read once per workgroup and used by all 256 rows whatever
// candidate they belong to - the prefix is never expanded over candidates (Sec. 4.2).
// Suffix part: each wavefront attends causally to the suffix K/V of the (one or few)
// candidates its rows belong to.  Both parts feed one online-softmax state per row (running
// max, running sum, unnormalised output), so the result is Eq. 2 over the concatenation
// [prefix ; own suffix] without that concatenation ever existing.
//
// Matrix-core formulation (v_mfma_f32_16x16x32_bf16, fp32 accumulate), transposed so that a
// lane owns a query column:
//     S^T[key][q] = sum_d K[key][d] * Q[q][d]        A = K tile (LDS),  B = Q (registers)
//     O^T[d][q]  += sum_key V[key][d] * P^T[key][q]  A = V^T (LDS, transposing read), B = P^T
// The accumulator layout of S^T (lane: column q = lane%16, rows 4*(lane/16)+t) is, up to a
// fixed permutation of the contraction index, the B-operand layout of the second product, so
// probabilities go from the first MFMA to the second through registers only; the same
// permutation is applied to the rows of V when its A fragments are read.
#include "pskv_internal.h"

namespace pskv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;                       // head dimension
constexpr int kRowBytes = kD * 2;             // one K/V/Q row in bf16
constexpr int kKT = 64;                       // prefix keys per LDS tile
constexpr int kNQ = 2;                        // 16-row query blocks per wavefront
constexpr int kNW = 8;                        // wavefronts per workgroup
constexpr int kWaveRows = 16 * kNQ;           // 32
constexpr int kMT = kNW * kWaveRows;          // 256 rows per workgroup
constexpr int kTileBytes = kKT * kRowBytes;   // 16 KB
constexpr int kSufKeys = 32;                  // suffix keys per step
constexpr int kScrBytes = kSufKeys * kRowBytes;
constexpr int kLdsBytes = 4 * kTileBytes + kNW * kScrBytes; // K,V double-buffered + V scratch
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) unsigned char lds_u8;

// Byte offset of 16-byte chunk `chunk` (0..15) of row `row` inside an LDS tile whose rows are
// 256 bytes: chunks are XOR-swizzled with the row number so that 16 rows read at the same
// logical chunk (K fragments) and 4 rows x 32 bytes read per 16 lanes (transposing V reads)
// both spread over all banks without padding.
__device__ inline unsigned swz(int row, int chunk) { return (unsigned)(row * kRowBytes + ((chunk ^ (row & 15)) << 4)); }

__device__ inline uintx4 ld_global16(const unsigned short *p) { return *reinterpret_cast<const uintx4 *>(p); }

__device__ inline bf16x8 as_bf16x8(uintx4 v)
{
    bf16x8 r;
    __builtin_memcpy(&r, &v, 16);
    return r;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Two fp32 -> packed bf16 (round to nearest even), as one 32-bit word.
__device__ inline unsigned pack_bf16(float lo, float hi)
{
    floatx2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    unsigned r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// Transposing LDS read: the 16 lanes of a group each name 8 bytes (4 bf16); lane t receives
// element (t % 4) of source lanes 4e + t/4, e = 0..3 - i.e. when lanes 4e..4e+3 name 16
// consecutive columns of row e, lane t gets column t of rows 0..3.
__device__ inline short4v lds_read_tr(lds_u8 *base, unsigned off)
{
    typedef short4v __attribute__((address_space(3))) * tr_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(base + off));
}

struct RowState {
    float m;      // running max of scaled scores, in log2 units
    float l;      // this lane's share of the running sum (lanes of one column hold 4 shares)
    floatx4 o[8]; // O^T accumulators: o[dt][t] = O^T[16*dt + 4*(lane/16) + t][lane % 16]
};

// Online-softmax update of one query block with NKT tiles of 16 keys whose masked scores
// (raw dot products, -inf where not visible) are in s.  Produces the P^T fragments for the
// second MFMA: fragment j covers tiles 2j and 2j+1.
template <int NKT>
__device__ inline void softmax_update(floatx4 (&s)[NKT], RowState &st, float c, bf16x8 (&pf)[NKT / 2])
{
    float tmax = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            tmax = fmaxf(tmax, s[kt][t]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mnew = fmaxf(st.m, tmax * c);
    const float msafe = mnew == -INFINITY ? 0.f : mnew; // row with nothing visible yet
    const float alpha = fast_exp2(st.m - msafe);
    float rs = 0.f;
#pragma unroll
    for (int j = 0; j < NKT / 2; ++j) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = fast_exp2(__builtin_fmaf(s[2 * j + e / 4][e % 4], c, -msafe));
            rs += p[e];
        }
        uintx4 w = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
        pf[j] = as_bf16x8(w);
    }
    st.l = st.l * alpha + rs;
    st.m = mnew;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) { // wave-uniform: skip when no max moved
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            st.o[dt] *= alpha;
    }
}

// O^T += V^T P^T for 32 keys held in rows [row_base, row_base+32) of the LDS tile `vt`.
// Contraction slot (lane group g, element e) stands for key 16*(e/4) + 4*g + e%4, the key the
// S^T accumulator holds at tile e/4, element e%4.
__device__ inline void pv_step(lds_u8 *vt, int row_base, int g, int c16, const bf16x8 (&pf)[kNQ],
                               const bool (&qbv)[kNQ], RowState (&st)[kNQ])
{
    const int r0 = row_base + 4 * g + (c16 >> 2);
    const int sub = (c16 & 1) * 8;
    const int chalf = (c16 & 3) >> 1;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        const int chunk = 2 * dt + chalf;
        short4v lo = lds_read_tr(vt, swz(r0, chunk) + sub);
        short4v hi = lds_read_tr(vt, swz(r0 + 16, chunk) + sub);
        short8v v8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 vf;
        __builtin_memcpy(&vf, &v8, 16);
#pragma unroll
        for (int qb = 0; qb < kNQ; ++qb)
            if (qbv[qb])
                st[qb].o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qb], st[qb].o[dt], 0, 0, 0);
    }
}

__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void mfma_stream_kernel(Args a)
{
    extern __shared__ __align__(16) unsigned char smem_generic[];
    lds_u8 *smem = (lds_u8 *)smem_generic;
    lds_u8 *kbuf = smem;                  // [2][kTileBytes]
    lds_u8 *vbuf = smem + 2 * kTileBytes; // [2][kTileBytes]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c16 = lane & 15;
    lds_u8 *scr = smem + 4 * kTileBytes + wave * kScrBytes;

    const int head = blockIdx.x % a.Hkv;
    const int mtile = blockIdx.x / a.Hkv;
    const int Mtot = a.B * a.S * a.G;
    const int r0 = mtile * kMT + wave * kWaveRows; // first stacked row of this wavefront
    const float c = a.scale * kLog2e;

    const unsigned short *qg = reinterpret_cast<const unsigned short *>(a.q);
    const unsigned short *ksg = reinterpret_cast<const unsigned short *>(a.ks) + (long long)head * a.ks_sh;
    const unsigned short *vsg = reinterpret_cast<const unsigned short *>(a.vs) + (long long)head * a.ks_sh;
    const unsigned short *kpg = reinterpret_cast<const unsigned short *>(a.kp) + (long long)head * a.kp_sh;
    const unsigned short *vpg = reinterpret_cast<const unsigned short *>(a.vp) + (long long)head * a.kp_sh;

    // ---- prefix tile staging (whole workgroup): 64 rows x 16 chunks = 2 chunks per thread ----
    uintx4 stk[2], stv[2];
    auto tile_gload = [&](int tile) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int cid = tid + 512 * u;
            const int row = cid >> 4, ch = cid & 15;
            const int key = tile * kKT + row;
            if (key < a.P) {
                const long long off = (long long)key * a.kp_sp + ch * 8;
                stk[u] = ld_global16(kpg + off);
                stv[u] = ld_global16(vpg + off);
            } else { // rows past the prefix: zeros (their scores are masked, their V must not be NaN)
                stk[u] = uintx4{0, 0, 0, 0};
                stv[u] = uintx4{0, 0, 0, 0};
            }
        }
    };
    auto tile_lstore = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int cid = tid + 512 * u;
            const int row = cid >> 4, ch = cid & 15;
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(kbuf + buf * kTileBytes + swz(row, ch)) = stk[u];
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(vbuf + buf * kTileBytes + swz(row, ch)) = stv[u];
        }
    };
    const int ntiles = (a.P + kKT - 1) / kKT;
    if (ntiles > 0)
        tile_gload(0);

    // ---- this lane's query rows: lane column c16 of each 16-row block ----
    int rb[kNQ], ri[kNQ];
    bool rin[kNQ], rvalid[kNQ], qbv[kNQ];
    bf16x8 qf[kNQ][4];
    long long orow[kNQ];
    int rh[kNQ];
#pragma unroll
    for (int qb = 0; qb < kNQ; ++qb) {
        const int r = r0 + 16 * qb + c16;
        rin[qb] = r < Mtot;
        const int rr = rin[qb] ? r : 0;
        const int tok = rr / a.G, gq = rr - tok * a.G;
        const int b = tok / a.S, i = tok - b * a.S;
        int len = a.len ? a.len[b] : a.S;
        len = len < 0 ? 0 : (len > a.S ? a.S : len);
        rb[qb] = b;
        ri[qb] = i;
        rh[qb] = head * a.G + gq;
        rvalid[qb] = rin[qb] && i < len;
        orow[qb] = (long long)b * a.o_sb + (long long)i * a.o_ss + (long long)rh[qb] * a.o_sh;
        const unsigned short *qrow = qg + (long long)b * a.q_sb + (long long)i * a.q_ss + (long long)rh[qb] * a.q_sh;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            qf[qb][ks] = as_bf16x8(rvalid[qb] ? ld_global16(qrow + 32 * ks + 8 * g) : uintx4{0, 0, 0, 0});
        qbv[qb] = __builtin_amdgcn_ballot_w64(rvalid[qb]) != 0; // block has at least one real row
    }
    const bool wave_active = qbv[0] || qbv[1];

    RowState st[kNQ];
#pragma unroll
    for (int qb = 0; qb < kNQ; ++qb) {
        st[qb].m = -INFINITY;
        st[qb].l = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            st[qb].o[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- suffix part first (its loads overlap the first prefix tile's) ----
    if (wave_active) {
        const int last_row = (r0 + kWaveRows - 1 < Mtot ? r0 + kWaveRows - 1 : Mtot - 1);
        const int tok_first = r0 / a.G, tok_last = last_row / a.G;
        const int b_first = tok_first / a.S, b_last = tok_last / a.S;
        for (int b = b_first; b <= b_last; ++b) { // wave-uniform
            int len = a.len ? a.len[b] : a.S;
            len = len < 0 ? 0 : (len > a.S ? a.S : len);
            len = __builtin_amdgcn_readfirstlane(len);
            const int i_lo = tok_first - b * a.S > 0 ? tok_first - b * a.S : 0;
            const int i_hi = tok_last - b * a.S < a.S - 1 ? tok_last - b * a.S : a.S - 1;
            const int kmax = i_hi < len - 1 ? i_hi : len - 1; // last suffix key any row here can see
            if (i_lo >= len || kmax < 0)
                continue;
            const unsigned short *kb = ksg + (long long)b * a.ks_sb;
            const unsigned short *vb = vsg + (long long)b * a.ks_sb;
            for (int k0 = 0; k0 <= kmax; k0 += kSufKeys) {
                // K fragments straight from global memory in A-operand layout
                uintx4 kf[2][4];
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    const int key = k0 + 16 * t2 + c16;
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        kf[t2][ks] = key <= kmax ? ld_global16(kb + (long long)key * a.ks_ss + 32 * ks + 8 * g)
                                                 : uintx4{0, 0, 0, 0};
                }
                // V rows to this wavefront's scratch tile (zeros past kmax)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int cid = lane + 64 * u;
                    const int row = cid >> 4, ch = cid & 15;
                    const int key = k0 + row;
                    uintx4 v = key <= kmax ? ld_global16(vb + (long long)key * a.ks_ss + ch * 8) : uintx4{0, 0, 0, 0};
                    *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(scr + swz(row, ch)) = v;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();

                bf16x8 pf[kNQ][1] = {};
#pragma unroll
                for (int qb = 0; qb < kNQ; ++qb) {
                    if (!qbv[qb])
                        continue;
                    floatx4 s[2];
#pragma unroll
                    for (int t2 = 0; t2 < 2; ++t2) {
                        s[t2] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks)
                            s[t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[t2][ks]), qf[qb][ks], s[t2], 0, 0, 0);
                        // causal + same-candidate mask
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const int key = k0 + 16 * t2 + 4 * g + t;
                            const bool vis = rb[qb] == b && key <= ri[qb];
                            s[t2][t] = vis ? s[t2][t] : -INFINITY;
                        }
                    }
                    softmax_update<2>(s, st[qb], c, pf[qb]);
                }
                bf16x8 pfj[kNQ] = {pf[0][0], pf[1][0]};
                pv_step(scr, 0, g, c16, pfj, qbv, st);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }

    // ---- prefix part: stream 64-key tiles through LDS, one barrier per tile ----
    if (ntiles > 0) {
        tile_lstore(0);
        __syncthreads();
    }
    for (int tile = 0; tile < ntiles; ++tile) {
        const int buf = tile & 1;
        if (tile + 1 < ntiles)
            tile_gload(tile + 1);
        if (wave_active) {
            lds_u8 *kt_base = kbuf + buf * kTileBytes;
            lds_u8 *vt_base = vbuf + buf * kTileBytes;
            const int nvalid = a.P - tile * kKT; // keys of this tile that exist (>= 64: all)
            bf16x8 pf[kNQ][2] = {};
            floatx4 s[kNQ][4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                for (int qb = 0; qb < kNQ; ++qb)
                    s[qb][kt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const uintx4 kraw = *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(
                        kt_base + swz(16 * kt + c16, g + 4 * ks));
                    const bf16x8 kfrag = as_bf16x8(kraw);
#pragma unroll
                    for (int qb = 0; qb < kNQ; ++qb)
                        if (qbv[qb])
                            s[qb][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfrag, qf[qb][ks], s[qb][kt], 0, 0, 0);
                }
            }
            if (nvalid < kKT) { // ragged last tile: keys past the prefix are not visible
#pragma unroll
                for (int qb = 0; qb < kNQ; ++qb)
#pragma unroll
                    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (16 * kt + 4 * g + t >= nvalid)
                                s[qb][kt][t] = -INFINITY;
            }
#pragma unroll
            for (int qb = 0; qb < kNQ; ++qb)
                if (qbv[qb])
                    softmax_update<4>(s[qb], st[qb], c, pf[qb]);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bf16x8 pfj[kNQ] = {pf[0][j], pf[1][j]};
                pv_step(vt_base, 32 * j, g, c16, pfj, qbv, st);
            }
        }
        if (tile + 1 < ntiles)
            tile_lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and store (Eq. 2's division by the softmax denominator) ----
    unsigned short *og = reinterpret_cast<unsigned short *>(a.out);
#pragma unroll
    for (int qb = 0; qb < kNQ; ++qb) {
        float l = st[qb].l;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (!rin[qb])
            continue;
        const bool ok = rvalid[qb];
        const float inv = ok ? 1.0f / l : 0.f;
        unsigned short *orp = og + orow[qb];
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            uintx2 w = {0u, 0u};
            if (ok) {
                w[0] = pack_bf16(st[qb].o[dt][0] * inv, st[qb].o[dt][1] * inv);
                w[1] = pack_bf16(st[qb].o[dt][2] * inv, st[qb].o[dt][3] * inv);
            }
            *reinterpret_cast<uintx2 *>(orp + 16 * dt + 4 * g) = w;
        }
        if (a.lse && g == 0)
            a.lse[((long long)rb[qb] * a.Hq + rh[qb]) * a.S + ri[qb]] =
                ok ? (st[qb].m + __builtin_log2f(l)) * kLn2 : -INFINITY;
    }
}

} // namespace

bool mfma_supported(const Args &a, int dtype)
{
    if (dtype != 1 || a.D != kD)
        return false;
    const long long rows = (long long)a.B * a.S * a.G;
    const long long blocks = ((rows + kMT - 1) / kMT) * a.Hkv;
    return rows <= 0x7fffffffLL - kMT && blocks <= 0x7fffffffLL;
}

hipError_t launch_mfma(const Args &a, hipStream_t stream)
{
    return resident_supported(a) ? launch_resident(a, stream) : launch_stream(a, stream);
}

hipError_t launch_stream(const Args &a, hipStream_t stream)
{
    static bool attr_set = false; // raising the dynamic LDS limit is idempotent; a race is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_stream_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    const long long rows = (long long)a.B * a.S * a.G;
    const unsigned blocks = (unsigned)(((rows + kMT - 1) / kMT) * a.Hkv);
    hipLaunchKernelGGL(mfma_stream_kernel, dim3(blocks), dim3(kNW * 64), kLdsBytes, stream, a);
    return hipGetLastError();
}

} // namespace pskv
