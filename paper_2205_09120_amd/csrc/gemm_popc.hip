// Tiled popcount GEMM kernels for gfx950 (binary / ternary / ternary-binary, Section III of the paper).
//
// Design (differs from the paper's NEON microkernels on purpose: those are built around 128-bit registers, 16-bit
// accumulators and reordered operand blocks; here the wavefront, its scalar register file and LDS set the shape):
//   * One operand ("S", the scalar side) is read with scalar loads straight into SGPRs: every lane of a
//     wavefront works on the same TS bit strings of S, so they cost no vector registers and no LDS traffic.
//   * The other operand ("V", the vector side) is staged through LDS once per workgroup and every lane owns
//     TV bit strings of it (lane, lane+64, ...).  A wave therefore computes a TS x (64*TV) block of products
//     and a workgroup of WAVES waves a (WAVES*TS) x (64*TV) block.
//   * Per 32 depth positions and output the VALU executes
//        BNN: x = s ^ v;                    acc += popcount(x)                     (2 instructions, eq. (6))
//        TNN: m = nz_s & nz_v; u = (neg_s ^ neg_v) & m;  M += popcount(m); U += popcount(u)     (4 instructions)
//        TBN: u = (neg_v ^ y_s) & nz_v;     U += popcount(u)   (+ a per-string popcount(nz_v))  (2 instructions)
//        TBN with the ternary operand on the scalar side (few ternary strings, so that lanes own binary strings):
//             t = nz_s & y_v; u = neg_s ^ t;  U += popcount(u)   (3 instructions: only one operand of an
//             instruction may come from a scalar register, and neg is a subset of nz, so (neg ^ y) & nz = (nz & y) ^ neg;
//             popcount(nz_s) is counted on the scalar ALU)
//     where nz = x+ | x- and neg = x-.  With P = popcount(z+), Q = popcount(z-) of eq. (7): M = P + Q and U = Q,
//     so C = M - 2U (TNN) and C = popcount(nz_v) - 2U (TBN) are the integers eq. (7) defines; the forms need
//     fewer instructions than evaluating z+ and z- separately because gfx950 has a three-input bit operation.
//   * Accumulators are 32-bit; the epilogue applies eq. (6) / (7) and writes int32 C, or, in the orientation where
//     lanes own rows of C, compares against per-row thresholds and writes the packed low-bit feature map directly.
//   * Workgroup ids are mapped to tiles XCD by XCD so that the workgroups sharing a V tile share an L2.
//
// The ternary planes are converted from the stored (x+, x-) pair to (nz, neg) while the tile is staged, so the
// packed format in memory stays the paper's encoding.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>
#include <string.h>

#include "lowbit_internal.h"

namespace lowbit {

namespace {

constexpr int kPadEntries = 4;  // LDS row padding, in entries
constexpr int kComputeUnits = 256;  // MI355X

template <int KIND> struct Traits;
template <> struct Traits<KIND_BNN> { static constexpr int SD = 2, VD = 2, ACC = 1; };
template <> struct Traits<KIND_TNN> { static constexpr int SD = 4, VD = 4, ACC = 2; };
template <> struct Traits<KIND_TBN> { static constexpr int SD = 2, VD = 4, ACC = 1; };  // S binary, V ternary
template <> struct Traits<KIND_TBN_SV> { static constexpr int SD = 4, VD = 2, ACC = 1; };  // S ternary, V binary

template <int D> struct Vec;
template <> struct Vec<2> { using type = uint2; };
template <> struct Vec<4> { using type = uint4; };

__device__ __forceinline__ uint2 zero_of(uint2) { return make_uint2(0u, 0u); }
__device__ __forceinline__ uint4 zero_of(uint4) { return make_uint4(0u, 0u, 0u, 0u); }

// stored (plus, minus) -> (nz, neg)
__device__ __forceinline__ uint4 to_nz_neg(uint4 e) { return make_uint4(e.x | e.z, e.y | e.w, e.z, e.w); }
__device__ __forceinline__ uint2 to_nz_neg(uint2 e) { return e; }

// The compiler re-associates the bit logic and splits popcount-accumulate into two instructions when it sees
// plain C, so the three hot instructions are pinned with inline assembly.  `s` operands live in SGPRs (one
// scalar source per VALU instruction is the limit of this ISA generation).
__device__ __forceinline__ uint32_t and_sv(uint32_t s, uint32_t v)
{
    uint32_t r;
    asm("v_and_b32 %0, %1, %2" : "=v"(r) : "s"(s), "v"(v));
    return r;
}
__device__ __forceinline__ uint32_t xor_sv(uint32_t s, uint32_t v)
{
    uint32_t r;
    asm("v_xor_b32 %0, %1, %2" : "=v"(r) : "s"(s), "v"(v));
    return r;
}
// (s ^ v) & m : three-input bit operation, truth table built from a=0xF0, b=0xCC, c=0xAA -> (a^b)&c = 0x28
__device__ __forceinline__ uint32_t xor_and_svv(uint32_t s, uint32_t v, uint32_t m)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28" : "=v"(r) : "s"(s), "v"(v), "v"(m));
    return r;
}
// acc += popcount(x) in one instruction
__device__ __forceinline__ void popc_acc(int32_t &acc, uint32_t x)
{
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

// SG depth words of an S string are fetched by one scalar load (SG*SD dwords, at most 16), so that a wave waits for
// scalar memory once per SG depth words instead of once per word: 2 or 4 words for the large tiles (bounded by the
// SGPR budget of TS = 8 strings), up to 16 dwords for the small, latency-bound tile.
template <int N> struct alignas(4) Words { uint32_t w[N]; };

template <int N> using IntC = std::integral_constant<int, N>;

// LDS needs of one workgroup tile, shared by the kernels below and the tile routine.
template <int KIND, int TV, int KG> struct TileLds {
    using VVec = typename Vec<Traits<KIND>::VD>::type;
    static constexpr int NV = 64 * TV;
    static constexpr int STRIDE = NV + kPadEntries;
    static constexpr int STAGE = KG * STRIDE;                     // entries of one staging buffer
    static constexpr int NNZ = KIND == KIND_TBN ? NV : 1;          // per-string non-zero counts (TBN only)
};

// One workgroup tile: S block sb, V block vb of the problem described by the arguments.  KW depth words are
// multiplied; consecutive strings lie ldk words apart (ldk = KW unless the launch splits the depth, in which case
// Sp / Vp already point at the first word of this workgroup's depth range and K counts the positions of that range).
// accum: the results are added to C with integer atomics (depth-split launches into a cleared C) instead of stored.  TRM selects where product
// (s, v) goes: 0 -> C[s*ldc + v], 1 -> C[v*ldc + s] (or the re-quantized output), 2 -> decided by tr_rt at run time
// (workgroup-uniform), for launches that mix both orientations.
template <int KIND, int TS, int TV, int WAVES, int KG, int SG, int TRM, bool CONV = false>
__device__ __forceinline__ void gemm_popc_tile(const uint32_t *__restrict__ Sp, const uint32_t *__restrict__ Vp,
                                               int rowsS, int rowsV, int KW, int ldk, int K,
                                               int32_t *__restrict__ C, int64_t ldc, int sb, int vb, bool tr_rt,
                                               bool c16, bool accum,
                                               const int32_t *__restrict__ q_lo, const int32_t *__restrict__ q_hi,
                                               uint64_t *__restrict__ q_out, int q_planes,
                                               typename TileLds<KIND, TV, KG>::VVec *lds_base, int32_t *nnz_lds,
                                               const Im2colGeom *cg = nullptr)
{
    using T = Traits<KIND>;
    constexpr int SD = T::SD, VD = T::VD;
    using SVec = typename Vec<SD>::type;
    using VVec = typename Vec<VD>::type;
    constexpr int NV = 64 * TV;
    constexpr int STRIDE = NV + kPadEntries;
    constexpr int UNITS = TV * KG;            // wave-wide loads per stage
    static_assert(UNITS % WAVES == 0, "stage units must divide among the waves");
    constexpr int UPW = UNITS / WAVES;        // per wave
    const bool tr = TRM == 2 ? tr_rt : (TRM == 1);

    VVec(*lds)[KG * STRIDE] = reinterpret_cast<VVec(*)[KG * STRIDE]>(lds_base);  // two staging buffers

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int s0 = (sb * WAVES + wave) * TS;
    const int v0 = vb * NV;

    const SVec *__restrict__ Sv = reinterpret_cast<const SVec *>(Sp);
    const VVec *__restrict__ Vv = reinterpret_cast<const VVec *>(Vp);

    // row pointers of this wave's S strings (clamped: out-of-range rows recompute the last row, never stored)
    const SVec *srow[TS];
#pragma unroll
    for (int i = 0; i < TS; ++i) {
        int r = s0 + i;
        r = r < rowsS ? r : rowsS - 1;
        srow[i] = Sv + (int64_t)r * ldk;
    }

    int32_t acc[T::ACC][TS][TV];
#pragma unroll
    for (int a = 0; a < T::ACC; ++a)
#pragma unroll
        for (int i = 0; i < TS; ++i)
#pragma unroll
            for (int t = 0; t < TV; ++t)
                acc[a][i][t] = 0;

    // stage bookkeeping: unit u = wave*UPW + j covers V strings vseg*64 + lane at depth word g
    VVec pre[UPW];
    // TBN needs the number of non-zeros of every V string (eq. (7)).  Every wave of the workgroup reads the same V
    // strings, so counting in the main loop would repeat the work WAVES times; instead each staged element is counted
    // once, by the lane that stages it, and the partial counts meet in LDS after the main loop.
    int32_t nnz_part[UPW];
    // TBN_SV: non-zero counts of this wave's S strings (the same in every lane)
    int32_t snnz[TS];
#pragma unroll
    for (int i = 0; i < TS; ++i)
        snnz[i] = 0;
    if constexpr (KIND == KIND_TBN) {
#pragma unroll
        for (int j = 0; j < UPW; ++j)
            nnz_part[j] = 0;
        for (int e = threadIdx.x; e < NV; e += 64 * WAVES)
            nnz_lds[e] = 0;
    }
    // Convolution (CONV): V string v is output pixel (b, oy, ox) and its depth word kg is channel word cw of the input
    // pixel under window tap (ky, kx), in the depth order (ky, kx, c) of the unrolled operand, or zero in the
    // padding -- the words are gathered from the channel-packed feature map while the tile is staged, the unrolled
    // operand is never written.  The units a thread stages are consecutive depth words of ONE V string (asserted
    // below), so the thread keeps one pixel: its window origin and the entry index of that origin in the map.  The tap
    // of the next depth word is wave-uniform and advances by KG words per stage without divisions.  When the channel
    // words per pixel are a multiple of KG, all words of a stage lie under one tap and share one bounds check and one
    // address (the vector ALU is what bounds this kernel, so address arithmetic per word would cost its share of it:
    // measured +10 % on the 3 x 3 x 512 layer, against +3 % this way).
    static_assert(!CONV || (UPW <= KG && KG % UPW == 0), "a thread's staging units must share a V string");
    int c_iy0 = 0, c_ix0 = 0, c_ky = 0, c_kx = 0, c_cw = 0;
    int64_t c_base = 0;
    bool c_ok = false, c_fast = false;
    if constexpr (CONV) {
        const int u0 = wave * UPW;
        const int vseg = u0 / KG, g0 = u0 % KG;
        const int v = v0 + vseg * 64 + lane;
        c_ok = v < rowsV;
        const int vv = c_ok ? v : 0;
        const int per = cg->OH * cg->OW;
        const int b = vv / per, rem = vv - b * per;
        const int oy = rem / cg->OW, ox = rem - oy * cg->OW;
        c_iy0 = oy * cg->sh - cg->ph;
        c_ix0 = ox * cg->sw - cg->pw;
        c_base = (((int64_t)b * cg->H + c_iy0) * cg->W + c_ix0) * cg->CW;  // may point outside the map; used in bounds only
        const int tap = g0 / cg->CW;
        c_cw = g0 - tap * cg->CW;
        c_ky = tap / cg->kw;
        c_kx = tap - c_ky * cg->kw;
        c_fast = cg->CW % KG == 0;
    }
    auto fetch = [&](int kg0) {
        if constexpr (CONV) {
            const int g0 = (wave * UPW) % KG;
            if (c_fast) {
                // one tap for the whole stage
                const int iy = c_iy0 + c_ky, ix = c_ix0 + c_kx;
                const bool in = c_ok && (unsigned)iy < (unsigned)cg->H && (unsigned)ix < (unsigned)cg->W;
                const VVec *src = Vv + c_base + ((int64_t)c_ky * cg->W + c_kx) * cg->CW + c_cw;
#pragma unroll
                for (int j = 0; j < UPW; ++j) {
                    VVec e = zero_of(VVec{});
                    if (in && kg0 + g0 + j < KW)
                        e = src[j];
                    pre[j] = e;
                }
                c_cw += KG;
                if (c_cw >= cg->CW) {
                    c_cw -= cg->CW;
                    if (++c_kx == cg->kw) {
                        c_kx = 0;
                        ++c_ky;
                    }
                }
            } else {
                // general case: walk the tap word by word (scalar state), one bounds check and address per word
                int ky = c_ky, kx = c_kx, cw = c_cw;
#pragma unroll
                for (int j = 0; j < UPW; ++j) {
                    const int iy = c_iy0 + ky, ix = c_ix0 + kx;
                    VVec e = zero_of(VVec{});
                    if (c_ok && kg0 + g0 + j < KW && (unsigned)iy < (unsigned)cg->H && (unsigned)ix < (unsigned)cg->W)
                        e = Vv[c_base + ((int64_t)ky * cg->W + kx) * cg->CW + cw];
                    pre[j] = e;
                    if (++cw == cg->CW) {
                        cw = 0;
                        if (++kx == cg->kw) {
                            kx = 0;
                            ++ky;
                        }
                    }
                }
                // the thread's first word of the next stage is KG words further down the depth
                c_cw += KG;
                while (c_cw >= cg->CW) {
                    c_cw -= cg->CW;
                    if (++c_kx == cg->kw) {
                        c_kx = 0;
                        ++c_ky;
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < UPW; ++j) {
                const int u = wave * UPW + j;
                const int vseg = u / KG, g = u % KG;
                const int v = v0 + vseg * 64 + lane;
                const int kg = kg0 + g;
                VVec e = zero_of(VVec{});
                if (v < rowsV && kg < KW)
                    e = Vv[(int64_t)v * ldk + kg];
                pre[j] = e;
            }
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < UPW; ++j) {
            const int u = wave * UPW + j;
            const int vseg = u / KG, g = u % KG;
            const VVec e = to_nz_neg(pre[j]);
            lds[buf][g * STRIDE + vseg * 64 + lane] = e;
            if constexpr (KIND == KIND_TBN) {
                popc_acc(nnz_part[j], e.x);
                popc_acc(nnz_part[j], e.y);
            }
        }
    };

    const int nchunks = (KW + KG - 1) / KG;
    fetch(0);
    commit(0);
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        const int kg0 = c * KG;
        if (c + 1 < nchunks)
            fetch(kg0 + KG);
        const int gmax = (KW - kg0) < KG ? (KW - kg0) : KG;
        auto body1 = [&](int g) __attribute__((always_inline)) {
            SVec sv[TS];
#pragma unroll
            for (int i = 0; i < TS; ++i)
                sv[i] = srow[i][kg0 + g];
            uint32_t snz0[TS], snz1[TS];
            if constexpr (KIND == KIND_TNN || KIND == KIND_TBN_SV) {
#pragma unroll
                for (int i = 0; i < TS; ++i) {
                    snz0[i] = sv[i].x | sv[i].z;
                    snz1[i] = sv[i].y | sv[i].w;
                    if constexpr (KIND == KIND_TBN_SV)
                        snnz[i] += __builtin_popcount(snz0[i]) + __builtin_popcount(snz1[i]);
                }
            }
            VVec bnext = lds[buf][g * STRIDE + lane];
#pragma unroll
            for (int t = 0; t < TV; ++t) {
                const VVec b = bnext;
                if (t + 1 < TV)
                    bnext = lds[buf][g * STRIDE + (t + 1) * 64 + lane];
                if constexpr (KIND == KIND_BNN) {
#pragma unroll
                    for (int i = 0; i < TS; ++i) {
                        popc_acc(acc[0][i][t], xor_sv(sv[i].x, b.x));
                        popc_acc(acc[0][i][t], xor_sv(sv[i].y, b.y));
                    }
                } else if constexpr (KIND == KIND_TNN) {
#pragma unroll
                    for (int i = 0; i < TS; ++i) {
                        const uint32_t m0 = and_sv(snz0[i], b.x), m1 = and_sv(snz1[i], b.y);
                        const uint32_t u0 = xor_and_svv(sv[i].z, b.z, m0), u1 = xor_and_svv(sv[i].w, b.w, m1);
                        popc_acc(acc[0][i][t], m0);
                        popc_acc(acc[1][i][t], u0);
                        popc_acc(acc[0][i][t], m1);
                        popc_acc(acc[1][i][t], u1);
                    }
                } else if constexpr (KIND == KIND_TBN) {
#pragma unroll
                    for (int i = 0; i < TS; ++i) {
                        popc_acc(acc[0][i][t], xor_and_svv(sv[i].x, b.z, b.x));
                        popc_acc(acc[0][i][t], xor_and_svv(sv[i].y, b.w, b.y));
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < TS; ++i) {
                        popc_acc(acc[0][i][t], xor_sv(sv[i].z, and_sv(snz0[i], b.x)));
                        popc_acc(acc[0][i][t], xor_sv(sv[i].w, and_sv(snz1[i], b.y)));
                    }
                }
            }
        };
        // SG depth words at a time: all scalar loads and all LDS reads of the batch are issued before the first use
        auto bodyN = [&](auto sgc, int g) __attribute__((always_inline)) {
            constexpr int SGN = decltype(sgc)::value;
            constexpr int NW = SGN * SD;
            static_assert(NW <= 16, "a scalar load fetches at most 16 dwords");
            Words<NW> sw[TS];
#pragma unroll
            for (int i = 0; i < TS; ++i)
                sw[i] = *reinterpret_cast<const Words<NW> *>(srow[i] + kg0 + g);
            VVec b[SGN][TV];
#pragma unroll
            for (int q = 0; q < SGN; ++q)
#pragma unroll
                for (int t = 0; t < TV; ++t)
                    b[q][t] = lds[buf][(g + q) * STRIDE + t * 64 + lane];
            if constexpr (KIND == KIND_TNN) {
                // The four instructions of a unit (one row, one V string, 32 depth positions) depend on each other:
                // and -> bitop3 -> count, and -> count.  Issued unit by unit, each waits for the one before it; here the
                // and of unit k+1 sits between the two counts of unit k and its bitop3 behind them, which measures 4-5 %
                // faster (register-only chains at four waves per SIMD, and this kernel on the 1024 x 50176 x 4608
                // problem: 761 -> 727 us).  Volatile: the compiler keeps this order.  The same treatment of the
                // two-instruction kinds (logic of unit k+1 in front of the count of unit k) measured 3-6 % SLOWER than
                // the compiler's own interleaving, so they keep the plain form below.
                auto &accr = acc;  // named here so that the generic lambda captures it
                constexpr int U = SGN * TV * TS * 2;
                uint32_t mm[2], uu[2];
                {
                    const uint32_t pw = sw[0].w[0], nw = sw[0].w[2];
                    asm volatile("v_and_b32 %0, %1, %2" : "=v"(mm[0]) : "s"(pw | nw), "v"(b[0][0].x));
                    asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28" : "=v"(uu[0]) : "s"(nw), "v"(b[0][0].z), "v"(mm[0]));
                }
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    // unit k = (depth word q, V string t, row i, half h), h fastest
                    const int i = (k >> 1) % TS, t = (k / (2 * TS)) % TV;
                    const int k1 = k + 1 < U ? k + 1 : k;
                    const int h = k1 & 1, i1 = (k1 >> 1) % TS, t1 = (k1 / (2 * TS)) % TV, q1 = k1 / (2 * TS * TV);
                    const uint32_t pw = sw[i1].w[q1 * 4 + h], nw = sw[i1].w[q1 * 4 + 2 + h];
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(accr[0][i][t]) : "v"(mm[k & 1]));
                    if (k + 1 < U)
                        asm volatile("v_and_b32 %0, %1, %2" : "=v"(mm[(k + 1) & 1]) : "s"(pw | nw), "v"(h ? b[q1][t1].y : b[q1][t1].x));
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(accr[1][i][t]) : "v"(uu[k & 1]));
                    if (k + 1 < U)
                        asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x28"
                                     : "=v"(uu[(k + 1) & 1])
                                     : "s"(nw), "v"(h ? b[q1][t1].w : b[q1][t1].z), "v"(mm[(k + 1) & 1]));
                }
            } else
#pragma unroll
            for (int q = 0; q < SGN; ++q)
#pragma unroll
                for (int t = 0; t < TV; ++t) {
                    const VVec bb = b[q][t];
                    if constexpr (KIND == KIND_BNN) {
#pragma unroll
                        for (int i = 0; i < TS; ++i) {
                            popc_acc(acc[0][i][t], xor_sv(sw[i].w[q * 2], bb.x));
                            popc_acc(acc[0][i][t], xor_sv(sw[i].w[q * 2 + 1], bb.y));
                        }
                    } else if constexpr (KIND == KIND_TBN) {
#pragma unroll
                        for (int i = 0; i < TS; ++i) {
                            popc_acc(acc[0][i][t], xor_and_svv(sw[i].w[q * 2], bb.z, bb.x));
                            popc_acc(acc[0][i][t], xor_and_svv(sw[i].w[q * 2 + 1], bb.w, bb.y));
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < TS; ++i) {
                            const uint32_t p0 = sw[i].w[q * 4], p1 = sw[i].w[q * 4 + 1];
                            const uint32_t n0 = sw[i].w[q * 4 + 2], n1 = sw[i].w[q * 4 + 3];
                            const uint32_t z0 = p0 | n0, z1 = p1 | n1;
                            if (t == 0)  // uniform values: counted once per string on the scalar ALU
                                snnz[i] += __builtin_popcount(z0) + __builtin_popcount(z1);
                            popc_acc(acc[0][i][t], xor_sv(n0, and_sv(z0, bb.x)));
                            popc_acc(acc[0][i][t], xor_sv(n1, and_sv(z1, bb.y)));
                        }
                    }
                }
        };
        // batches of SG depth words, then the remainder in halving batch sizes, then single words
        int g = 0;
        if constexpr (SG > 1) {
            for (; g + SG <= gmax; g += SG)
                bodyN(IntC<SG>{}, g);
            if constexpr (SG >= 8) {
                if (g + 4 <= gmax) {
                    bodyN(IntC<4>{}, g);
                    g += 4;
                }
            }
            if constexpr (SG >= 4) {
                if (g + 2 <= gmax) {
                    bodyN(IntC<2>{}, g);
                    g += 2;
                }
            }
        }
        for (; g < gmax; ++g)
            body1(g);
        if (c + 1 < nchunks)
            commit(buf ^ 1);
        __syncthreads();
    }

    int32_t nnz[TV];
    if constexpr (KIND == KIND_TBN) {
        // the main loop ended with a barrier, which also ordered the zero-fill of nnz_lds before these additions
#pragma unroll
        for (int j = 0; j < UPW; ++j) {
            const int vseg = (wave * UPW + j) / KG;
            atomicAdd(&nnz_lds[vseg * 64 + lane], nnz_part[j]);
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TV; ++t)
            nnz[t] = nnz_lds[t * 64 + lane];
    }

    // epilogue: eq. (6) / (7), then either the int32 store or (transposed orientation only) re-quantization
#pragma unroll
    for (int t = 0; t < TV; ++t) {
        const int v = v0 + t * 64 + lane;
        int32_t out[TS];
#pragma unroll
        for (int i = 0; i < TS; ++i) {
            if constexpr (KIND == KIND_BNN)
                out[i] = K - 2 * acc[0][i][t];
            else if constexpr (KIND == KIND_TNN)
                out[i] = acc[0][i][t] - 2 * acc[1][i][t];
            else if constexpr (KIND == KIND_TBN)
                out[i] = nnz[t] - 2 * acc[0][i][t];
            else
                out[i] = snnz[i] - 2 * acc[0][i][t];
        }
        if (tr) {
            if (q_out != nullptr) {
                // Lanes own 64 consecutive V rows (channels), so a wave-wide vote on "c > hi" / "c < lo" is exactly one
                // 64-bit depth word of the packed output string of S row s0+i.  Lane 0 stores it.
                const bool live = v < rowsV;
                const int32_t lo = live ? q_lo[v] : 0, hi = (live && q_planes == 2) ? q_hi[v] : 0;
                const int64_t mw = ((int64_t)rowsV + 63) / 64;
#pragma unroll
                for (int i = 0; i < TS; ++i) {
                    const uint64_t minus = __ballot(live && out[i] < lo);
                    const uint64_t plus = __ballot(live && out[i] > hi && !(out[i] < lo));
                    if (lane == 0 && s0 + i < rowsS && (v0 >> 6) + t < mw) {
                        const int64_t word = (int64_t)(s0 + i) * mw + (v0 >> 6) + t;
                        if (q_planes == 2) {
                            q_out[word * 2] = plus;
                            q_out[word * 2 + 1] = minus;
                        } else {
                            q_out[word] = minus;
                        }
                    }
                }
                continue;
            }
        }
        if (accum && tr) {
            // lanes own rows of C here: adding straight from the registers would touch 64 rows per instruction.  The
            // workgroup's (WAVES*TS) x 64 results go through LDS (the tile buffers are free after the main loop), so
            // that consecutive threads add to consecutive columns of a row.
            constexpr int SW = WAVES * TS;
            int32_t *stage = reinterpret_cast<int32_t *>(lds_base);
            static_assert(SW * 64 * 4 <= (int)sizeof(VVec) * 2 * KG * STRIDE, "staging must fit the tile buffers");
            __syncthreads();  // every wave is done with the tile buffers (and with the staging of the previous t)
#pragma unroll
            for (int i = 0; i < TS; ++i)
                stage[lane * SW + wave * TS + i] = out[i];
            __syncthreads();
            for (int e = threadIdx.x; e < SW * 64; e += 64 * WAVES) {
                const int vl = e / SW, sl = e - vl * SW;
                const int vv = v0 + t * 64 + vl, ss = sb * SW + sl;
                if (vv < rowsV && ss < rowsS)
                    atomicAdd(C + (int64_t)vv * ldc + ss, stage[e]);
            }
            continue;
        }
        if constexpr ((WAVES * TS + 4) * 64 * 4 <= (int)sizeof(VVec) * 2 * KG * STRIDE && TRM != 0) {
            if (tr && !accum && !c16) {
                // Lanes own rows of C here and hold TS consecutive columns of them: stored from the registers, every
                // lane would write a 4 * TS byte piece of a line that other waves complete.  The workgroup's
                // (WAVES*TS) x 64 results go through LDS instead (the tile buffers are free after the main loop) and
                // leave as whole rows of the tile: 16 bytes per thread, consecutive threads on consecutive columns,
                // written through the L2 when the launch is large enough for the write-back at its end to matter
                // (measured: 1024 x 12544 x 4608 TBN 121 -> 111 us, 512 x 12544 x 2304 39.1 -> 34.9 us; launches of a few
                // workgroups are 0.1 - 0.3 us faster with plain stores).
                constexpr int SW = WAVES * TS, PITCH = SW + 4, CPR = SW / 4;
                const bool through = gridDim.x >= 2 * kComputeUnits;
                int32_t *stage = reinterpret_cast<int32_t *>(lds_base);
                __syncthreads();  // every wave is done with the tile buffers (and with the staging of the previous t)
                if constexpr (TS % 4 == 0) {
#pragma unroll
                    for (int i = 0; i < TS; i += 4)
                        *reinterpret_cast<int4 *>(stage + lane * PITCH + wave * TS + i) =
                            make_int4(out[i], out[i + 1], out[i + 2], out[i + 3]);
                } else {
#pragma unroll
                    for (int i = 0; i < TS; ++i)
                        stage[lane * PITCH + wave * TS + i] = out[i];
                }
                __syncthreads();
                for (int e = threadIdx.x; e < 64 * CPR; e += 64 * WAVES) {
                    const int vl = e / CPR, ch = e - vl * CPR;
                    const int vv = v0 + t * 64 + vl, ss = sb * SW + ch * 4;
                    if (vv < rowsV && ss < rowsS) {
                        const int4 q = *reinterpret_cast<const int4 *>(stage + vl * PITCH + ch * 4);
                        int32_t *dst = C + (int64_t)vv * ldc + ss;
                        if (ss + 4 <= rowsS) {
                            if (through)
                                store_through16(dst, q.x, q.y, q.z, q.w);
                            else
                                __builtin_memcpy(dst, &q, 16);  // no 16-byte alignment needed
                        } else {
                            dst[0] = q.x;
                            if (ss + 1 < rowsS)
                                dst[1] = q.y;
                            if (ss + 2 < rowsS)
                                dst[2] = q.z;
                        }
                    }
                }
                continue;
            }
        }
        if (v < rowsV) {
            if (accum) {
#pragma unroll
                for (int i = 0; i < TS; ++i)
                    if (s0 + i < rowsS)
                        atomicAdd(C + (int64_t)(s0 + i) * ldc + v, out[i]);
                continue;
            }
            if (c16) {
                // 16-bit C (the accumulator width of Section III; the host has checked K <= 32767, so |c| fits)
                int16_t *C16 = reinterpret_cast<int16_t *>(C);
                if (!tr) {
#pragma unroll
                    for (int i = 0; i < TS; ++i)
                        if (s0 + i < rowsS)
                            C16[(int64_t)(s0 + i) * ldc + v] = (int16_t)out[i];
                } else {
                    int16_t *crow = C16 + (int64_t)v * ldc + s0;
                    bool done = false;
                    if constexpr (TS % 4 == 0) {
                        if (s0 + TS <= rowsS) {
#pragma unroll
                            for (int i = 0; i < TS; i += 4) {
                                const int2 q = make_int2((out[i] & 0xffff) | (out[i + 1] << 16),
                                                         (out[i + 2] & 0xffff) | (out[i + 3] << 16));
                                __builtin_memcpy(crow + i, &q, 8);  // no 8-byte alignment needed
                            }
                            done = true;
                        }
                    }
                    if (!done) {
#pragma unroll
                        for (int i = 0; i < TS; ++i)
                            if (s0 + i < rowsS)
                                crow[i] = (int16_t)out[i];
                    }
                }
                continue;
            }
            if (!tr) {
#pragma unroll
                for (int i = 0; i < TS; ++i)
                    if (s0 + i < rowsS)
                        store_through(C + (int64_t)(s0 + i) * ldc + v, out[i]);
            } else {
                int32_t *crow = C + (int64_t)v * ldc + s0;
                if constexpr (TS % 4 == 0) {
                    if (s0 + TS <= rowsS) {
                        // (instances whose tile buffers cannot hold the staged results, and the 16-bit path above,
                        // store from the registers.)  128-bit stores through memcpy: they need no 16-byte alignment
                        // (odd ldc, odd N).  Plain stores: a lane writes 16 bytes of a line that other waves complete
                        // later, and written through, those pieces would reach memory one by one (measured 13 % slower
                        // on 1024 x 50176 x 4608); the L2 has to merge them.
#pragma unroll
                        for (int i = 0; i < TS; i += 4) {
                            const int4 q = make_int4(out[i], out[i + 1], out[i + 2], out[i + 3]);
                            __builtin_memcpy(crow + i, &q, 16);
                        }
                        continue;
                    }
                }
#pragma unroll
                for (int i = 0; i < TS; ++i)
                    if (s0 + i < rowsS)
                        crow[i] = out[i];
            }
        }
    }
}

template <int KIND, int TS, int TV, int WAVES, int KG, int SG, bool TR>
__global__ __launch_bounds__(64 * WAVES) void gemm_popc_kernel(const uint32_t *__restrict__ Sp,
                                                               const uint32_t *__restrict__ Vp, int rowsS, int rowsV,
                                                               int KW, int K, int32_t *__restrict__ C, int64_t ldc,
                                                               int nSB, int nVB, int tiles_per_xcd, int vb_fastest,
                                                               int c16, const int32_t *__restrict__ q_lo,
                                                               const int32_t *__restrict__ q_hi,
                                                               uint64_t *__restrict__ q_out, int q_planes)
{
    using L = TileLds<KIND, TV, KG>;
    __shared__ typename L::VVec lds[2 * L::STAGE];
    __shared__ int32_t nnz_lds[L::NNZ];

    // XCD-aware tile order: consecutive workgroup ids go to different XCDs, so give each XCD a contiguous
    // range of tiles.  Within it the tiles that share a block of the LARGER operand are adjacent, so that operand is
    // streamed from HBM once and the smaller one stays in that XCD's L2: the S blocks of one V tile when V is the
    // larger operand, the V blocks of one S block (vb_fastest) when S is.
    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nSB * nVB)
        return;
    int vb, sb;
    if (vb_fastest) {
        sb = idx / nVB;
        vb = idx - sb * nVB;
    } else {
        vb = idx / nSB;
        sb = idx - vb * nSB;
    }
    gemm_popc_tile<KIND, TS, TV, WAVES, KG, SG, TR ? 1 : 0>(Sp, Vp, rowsS, rowsV, KW, KW, K, C, ldc, sb, vb, TR,
                                                            c16 != 0, false, q_lo, q_hi, q_out, q_planes, lds, nnz_lds);
}

// Convolution as an implicit product: the kernel above with the V operand gathered from the channel-packed feature
// map (see the tile routine); A (the filters) is on the scalar side, C is M x N row-major with N = batch * OH * OW.
template <int KIND, int TS, int TV, int WAVES, int KG, int SG>
__global__ __launch_bounds__(64 * WAVES) void gemm_popc_conv_kernel(const uint32_t *__restrict__ Sp,
                                                                    const uint32_t *__restrict__ Fp, int rowsS, int rowsV,
                                                                    int KW, int K, int32_t *__restrict__ C, int64_t ldc,
                                                                    int nSB, int nVB, int tiles_per_xcd, int vb_fastest,
                                                                    const Im2colGeom geom)
{
    using L = TileLds<KIND, TV, KG>;
    __shared__ typename L::VVec lds[2 * L::STAGE];
    __shared__ int32_t nnz_lds[L::NNZ];
    const int bid = blockIdx.x;
    const int idx = (bid & 7) * tiles_per_xcd + (bid >> 3);
    if ((bid >> 3) >= tiles_per_xcd || idx >= nSB * nVB)
        return;
    int vb, sb;
    if (vb_fastest) {
        sb = idx / nVB;
        vb = idx - sb * nVB;
    } else {
        vb = idx / nSB;
        sb = idx - vb * nSB;
    }
    gemm_popc_tile<KIND, TS, TV, WAVES, KG, SG, 0, true>(Sp, Fp, rowsS, rowsV, KW, KW, K, C, ldc, sb, vb, false, false,
                                                         false, nullptr, nullptr, nullptr, 0, lds, nnz_lds, &geom);
}

template <int KIND, int TS, int TV, int WAVES, int KG, int SG>
hipError_t launch_conv(const GemmArgs &a, const Im2colGeom &g)
{
    if constexpr (KIND == KIND_BNN || KIND == KIND_TNN) {
        const int nSB = (a.rowsS + WAVES * TS - 1) / (WAVES * TS);
        const int nVB = (a.rowsV + 64 * TV - 1) / (64 * TV);
        const int64_t tiles = (int64_t)nSB * nVB;
        const int tiles_per_xcd = (int)((tiles + 7) / 8);
        const int64_t grid = (int64_t)tiles_per_xcd * 8;
        if (grid > 0x7fffffffLL)
            return hipErrorInvalidConfiguration;
        // the feature map is the smaller operand whenever the window has more than one tap: walk the S blocks of
        // one V tile first, as for a materialised operand
        hipLaunchKernelGGL((gemm_popc_conv_kernel<KIND, TS, TV, WAVES, KG, SG>), dim3((unsigned)grid), dim3(64 * WAVES),
                           0, a.stream, a.Sp, a.Vp, a.rowsS, a.rowsV, a.KW, a.K, a.C, a.ldc, nSB, nVB, tiles_per_xcd, 0,
                           g);
        return hipGetLastError();
    } else {
        return hipErrorNotSupported;  // the gathered operand must be on the vector side
    }
}

// Grouped launch: many independent small problems in one grid.  The table (built on the host by plan_group) maps
// each workgroup id to a problem record and the record gives the tile's place inside that problem.
template <int KIND, int TS, int TV, int WAVES, int KG, int SG>
__global__ __launch_bounds__(64 * WAVES) void gemm_group_kernel(const GroupHeader *__restrict__ table, uint32_t count)
{
    using L = TileLds<KIND, TV, KG>;
    __shared__ typename L::VVec lds[2 * L::STAGE];
    __shared__ int32_t nnz_lds[L::NNZ];

    // A table that was planned for another kind, problem count or grid is not read any further.
    const uint32_t bid = blockIdx.x;
    if (table->magic != kGroupMagic || table->kind != (uint32_t)KIND || table->count != count ||
        table->workgroups != gridDim.x)
        return;
    const GroupRecord *__restrict__ recs = reinterpret_cast<const GroupRecord *>(table + 1);
    const uint32_t *__restrict__ owner = reinterpret_cast<const uint32_t *>(recs + count);
    const uint32_t p = owner[bid];
    if (p >= count)
        return;
    const GroupRecord r = recs[p];
    const int local = (int)(bid - r.tile0);
    const int vb = local / r.nSB, sb = local - vb * r.nSB;
    gemm_popc_tile<KIND, TS, TV, WAVES, KG, SG, 2>(r.Sp, r.Vp, r.rowsS, r.rowsV, r.KW, r.KW, r.K, r.C, r.ldc, sb, vb,
                                                   r.transposed != 0, false, false, nullptr, nullptr, nullptr, 0, lds,
                                                   nnz_lds);
}

// Depth-split launch for products of few tiles and a long depth: workgroup (tile, z) multiplies depth words
// [z * words_per_split, ...) of its tile and adds the partial results to C, which a fill kernel cleared before.
// Exact in any order: the partial results of eq. (6) / (7) over disjoint depth ranges are integers that add up to C
// (eq. (6): K - 2 * popcount over a range counts that range's positions).
template <int KIND, int TS, int TV, int WAVES, int KG, int SG>
__global__ __launch_bounds__(64 * WAVES) void gemm_popc_splitk_kernel(const uint32_t *__restrict__ Sp,
                                                                      const uint32_t *__restrict__ Vp, int rowsS,
                                                                      int rowsV, int KW, int K, int32_t *__restrict__ C,
                                                                      int64_t ldc, int nSB, int transposed,
                                                                      int words_per_split)
{
    using L = TileLds<KIND, TV, KG>;
    using T = Traits<KIND>;
    __shared__ typename L::VVec lds[2 * L::STAGE];
    __shared__ int32_t nnz_lds[L::NNZ];
    const int tile = blockIdx.x, z = blockIdx.y;
    const int vb = tile / nSB, sb = tile - vb * nSB;
    const int kw0 = z * words_per_split;
    const int kw1 = kw0 + words_per_split < KW ? kw0 + words_per_split : KW;
    if (kw0 >= kw1)
        return;
    const int k_end = kw1 * 64 < K ? kw1 * 64 : K;
    gemm_popc_tile<KIND, TS, TV, WAVES, KG, SG, 2>(Sp + (int64_t)kw0 * T::SD, Vp + (int64_t)kw0 * T::VD, rowsS, rowsV,
                                                   kw1 - kw0, KW, k_end - kw0 * 64, C, ldc, sb, vb, transposed != 0,
                                                   false, true, nullptr, nullptr, nullptr, 0, lds, nnz_lds);
}

// zeroes the M x N part of C (row = blockIdx.y); the padding between N and ldc is left alone
__global__ __launch_bounds__(256) void clear_c_kernel(int32_t *__restrict__ C, int64_t ldc, int64_t N)
{
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n < N)
        C[(int64_t)blockIdx.y * ldc + n] = 0;
}

template <int KIND, int TS, int TV, int WAVES, int KG, int SG>
hipError_t launch_splitk(const GemmArgs &a, bool transposed, int nsplit)
{
    const int nSB = (a.rowsS + WAVES * TS - 1) / (WAVES * TS);
    const int nVB = (a.rowsV + 64 * TV - 1) / (64 * TV);
    const int64_t tiles = (int64_t)nSB * nVB;
    const int wps = (a.KW + nsplit - 1) / nsplit;
    const int nz = (a.KW + wps - 1) / wps;
    const int64_t M = transposed ? a.rowsV : a.rowsS, N = transposed ? a.rowsS : a.rowsV;
    if (tiles > 0x7fffffffLL || nz > 65535 || M > 65535)
        return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(clear_c_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)M), dim3(256), 0, a.stream, a.C, a.ldc, N);
    const hipError_t ec = hipGetLastError();
    if (ec != hipSuccess)  // without the cleared C the partial sums must not be added
        return ec;
    hipLaunchKernelGGL((gemm_popc_splitk_kernel<KIND, TS, TV, WAVES, KG, SG>), dim3((unsigned)tiles, (unsigned)nz),
                       dim3(64 * WAVES), 0, a.stream, a.Sp, a.Vp, a.rowsS, a.rowsV, a.KW, a.K, a.C, a.ldc, nSB,
                       transposed ? 1 : 0, wps);
    return hipGetLastError();
}

template <int KIND, int TS, int TV, int WAVES, int KG, int SG, bool TR>
hipError_t launch(const GemmArgs &a)
{
    const int nSB = (a.rowsS + WAVES * TS - 1) / (WAVES * TS);
    const int nVB = (a.rowsV + 64 * TV - 1) / (64 * TV);
    const int64_t tiles = (int64_t)nSB * nVB;
    const int tiles_per_xcd = (int)((tiles + 7) / 8);
    const int64_t grid = (int64_t)tiles_per_xcd * 8;
    if (grid > 0x7fffffffLL)
        return hipErrorInvalidConfiguration;
    // bytes per string: S strings have Traits::SD dwords per depth word, V strings Traits::VD
    const int vb_fastest = (int64_t)a.rowsS * Traits<KIND>::SD > (int64_t)a.rowsV * Traits<KIND>::VD;
    hipLaunchKernelGGL((gemm_popc_kernel<KIND, TS, TV, WAVES, KG, SG, TR>), dim3((unsigned)grid), dim3(64 * WAVES), 0,
                       a.stream, a.Sp, a.Vp, a.rowsS, a.rowsV, a.KW, a.K, a.C, a.ldc, nSB, nVB, tiles_per_xcd, vb_fastest,
                       a.c16, a.q_lo, a.q_hi, a.q_out, a.q_planes);
    return hipGetLastError();
}

#define LB_VARIANT(RANK, KIND, TS, TV, WAVES, KG, SG)                                               \
    {#KIND " ts" #TS " tv" #TV " w" #WAVES " kg" #KG " sg" #SG, RANK, TS * WAVES, 64 * TV,           \
     &launch<KIND, TS, TV, WAVES, KG, SG, false>, &launch<KIND, TS, TV, WAVES, KG, SG, true>, 0, 0,  \
     &launch_conv<KIND, TS, TV, WAVES, KG, SG>}
// ranked instance with conditions of its own: at least MIN_KW depth words and WANTED workgroups
#define LB_VARIANT_IF(RANK, MIN_KW, WANTED, KIND, TS, TV, WAVES, KG, SG)                            \
    {#KIND " ts" #TS " tv" #TV " w" #WAVES " kg" #KG " sg" #SG, RANK, TS * WAVES, 64 * TV,           \
     &launch<KIND, TS, TV, WAVES, KG, SG, false>, &launch<KIND, TS, TV, WAVES, KG, SG, true>, 0, MIN_KW, \
     &launch_conv<KIND, TS, TV, WAVES, KG, SG>, WANTED}
// latency-bound instance: taken for problems of at most SMALL_MAX tiles of 16 x 64 and at least MIN_KW depth words
#define LB_SMALL(SMALL_MAX, MIN_KW, KIND, TS, TV, WAVES, KG, SG)                                    \
    {#KIND " ts" #TS " tv" #TV " w" #WAVES " kg" #KG " sg" #SG, 0, TS * WAVES, 64 * TV,              \
     &launch<KIND, TS, TV, WAVES, KG, SG, false>, &launch<KIND, TS, TV, WAVES, KG, SG, true>, SMALL_MAX, MIN_KW, \
     &launch_conv<KIND, TS, TV, WAVES, KG, SG>}

// rank: preference of the shape-based selection (the highest rank wins among the variants that yield enough
// workgroups, otherwise the ranked variant with the most workgroups; 0 = only reachable through lb_set_variant).
// The first row of each table is the small-problem instance: 4 x 64 outputs per wave and scalar loads of 16 dwords.
// The LB_SMALL rows serve problems of a few hundred tiles, which are bound by the latency of their few dependent
// memory round trips rather than by throughput: 1 or 2 strings per wave and 8 waves per workgroup put more waves
// on every SIMD to overlap those round trips (measured 1.05-1.6x over the first row on such shapes; the limits
// come from a sweep over 64..512 x 64..3136 x 256..2304).  A row may repeat an instance with another condition.
const GemmVariant kBnn[] = {
    LB_VARIANT(1, KIND_BNN, 4, 1, 4, 16, 8),
    LB_VARIANT(2, KIND_BNN, 8, 1, 4, 8, 4),
    LB_VARIANT(5, KIND_BNN, 8, 2, 8, 8, 4),
    LB_VARIANT(0, KIND_BNN, 8, 4, 8, 8, 4),
    LB_VARIANT(3, KIND_BNN, 8, 2, 4, 8, 4),
    LB_VARIANT(0, KIND_BNN, 16, 2, 4, 8, 2),
    LB_VARIANT(0, KIND_BNN, 8, 2, 4, 8, 1),
    // 32 x 128 tile with eight waves of four rows (see the ternary table): for products too small for the 64 x 128
    // tile (512 x 8192 x 2304: 23.9 -> 21.7 us, 512 x 4096 x 2304: 15.3 -> 13.1 us, 2048 x 1024 x 4608: 23.9 -> 22.2 us)
    LB_VARIANT_IF(4, 32, 600, KIND_BNN, 4, 2, 8, 8, 4),
    LB_SMALL(64, 0, KIND_BNN, 1, 1, 4, 16, 8),
    LB_SMALL(160, 0, KIND_BNN, 1, 1, 8, 16, 8),
    LB_SMALL(300, 18, KIND_BNN, 1, 1, 8, 16, 8),
    LB_SMALL(600, 0, KIND_BNN, 2, 1, 8, 16, 8),
    LB_SMALL(1200, 0, KIND_BNN, 4, 1, 8, 16, 8),
};
const GemmVariant kTnn[] = {
    LB_VARIANT(1, KIND_TNN, 4, 1, 4, 16, 4),
    LB_VARIANT(2, KIND_TNN, 8, 1, 4, 8, 2),
    LB_VARIANT(3, KIND_TNN, 8, 2, 4, 4, 2),
    LB_VARIANT(4, KIND_TNN, 8, 4, 4, 4, 2),
    LB_VARIANT(0, KIND_TNN, 8, 4, 4, 4, 1),
    LB_VARIANT(0, KIND_TNN, 8, 4, 4, 2, 1),
    LB_VARIANT(0, KIND_TNN, 8, 4, 8, 4, 2),
    // 32 x 128 tile with eight waves of four rows: two waves of a workgroup on every SIMD, so that a workgroup keeps
    // its SIMDs fed on its own when the launch drains and fewer of them are resident; half the accumulators per wave.
    // Measured against the instances above: 1024 x 50176 x 4608 726 -> 719 us, 1024 x 12544 x 4608 203 -> 196 us,
    // 512 x 12544 x 2304 61 -> 59 us; shallow products (18 depth words: three stages of 8, 8, 2) are slower with it.
    LB_VARIANT_IF(6, 32, 1024, KIND_TNN, 4, 2, 8, 8, 4),
    // the same on a 32 x 64 tile, for products that yield fewer than 1024 of the tiles above (1024 x 3136 x 9216:
    // 130 -> 116 us, 512 x 6272 x 4608: 67.5 -> 61.2 us, 384 x 6272 x 3456: 40.1 -> 36.0 us)
    LB_VARIANT_IF(5, 32, 1024, KIND_TNN, 4, 1, 8, 16, 4),
    LB_SMALL(300, 0, KIND_TNN, 1, 1, 8, 16, 4),
    LB_SMALL(600, 0, KIND_TNN, 2, 1, 8, 16, 4),
    LB_SMALL(1200, 0, KIND_TNN, 4, 1, 8, 16, 4),
};
const GemmVariant kTbn[] = {
    LB_VARIANT(1, KIND_TBN, 4, 1, 4, 16, 8),
    LB_VARIANT_IF(2, 0, 1024, KIND_TBN, 8, 1, 4, 8, 4),  // from 1024 tiles (384 x 6272 x 3456: 27.6 -> 24.5 us)
    LB_VARIANT_IF(3, 0, 1024, KIND_TBN, 8, 2, 8, 8, 4),  // eight waves: half the workgroups of a four-wave tile fill the device
    LB_VARIANT(4, KIND_TBN, 8, 4, 8, 4, 1),
    LB_VARIANT(0, KIND_TBN, 8, 4, 4, 4, 4),
    LB_VARIANT(0, KIND_TBN, 8, 2, 4, 8, 4),
    LB_SMALL(64, 0, KIND_TBN, 1, 1, 4, 16, 8),
    LB_SMALL(160, 0, KIND_TBN, 1, 1, 8, 16, 8),
    LB_SMALL(300, 18, KIND_TBN, 1, 1, 8, 16, 8),
    LB_SMALL(1800, 18, KIND_TBN, 4, 1, 8, 16, 8),
};

// ternary operand on the scalar side: the scalar loads are those of the TNN instances
const GemmVariant kTbnSv[] = {
    LB_VARIANT(1, KIND_TBN_SV, 4, 1, 4, 16, 4),
    LB_VARIANT(2, KIND_TBN_SV, 8, 1, 4, 8, 2),
    LB_VARIANT(3, KIND_TBN_SV, 8, 2, 4, 4, 2),
    LB_SMALL(300, 0, KIND_TBN_SV, 1, 1, 8, 16, 4),
    LB_SMALL(600, 0, KIND_TBN_SV, 2, 1, 8, 16, 4),
    LB_SMALL(1200, 0, KIND_TBN_SV, 4, 1, 8, 16, 4),
};

// ---- launch table held by the library, for callers that cannot allocate device memory ----
//
// `scratch` is one table-sized array per GPU (each device that loads the code object holds its own copy until the
// process ends).  In host code the array's name is only a handle for hipGetSymbolAddress: the device address it yields
// is looked up once per device, with that device current, and used from then on wherever host code names the memory.
static __device__ __align__(256) unsigned char scratch[kGroupStaticBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

hipError_t group_scratch_ptr(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= kMaxDevices)
        return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return e;
        if (p == nullptr)
            return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
    }
    *out = p;
    return hipSuccess;
}

// A piece of the host-built table travels to the device inside the kernel arguments (copied by the runtime when the
// launch is enqueued, so the host table may be reused or freed right after the call, and the launch can be captured).
struct TableChunk {
    uint4 q[kGroupChunkBytes / 16];
};
__global__ __launch_bounds__(kGroupChunkBytes / 16) void group_table_upload_kernel(uint4 *__restrict__ dst,
                                                                                  const TableChunk chunk, int n16)
{
    const int i = threadIdx.x;
    if (i < n16)
        dst[i] = chunk.q[i];
}

}  // namespace

hipError_t launch_gemm_group_static(int kind, const void *table_host, size_t table_bytes, uint32_t count,
                                    uint32_t workgroups, hipStream_t stream)
{
    if (table_bytes == 0 || table_bytes % 16 != 0 || table_bytes > kGroupStaticBytes)
        return hipErrorInvalidValue;
    void *dev_table = nullptr;
    hipError_t e = group_scratch_ptr(&dev_table);
    if (e != hipSuccess)
        return e;
    const unsigned char *src = static_cast<const unsigned char *>(table_host);
    for (size_t off = 0; off < table_bytes; off += kGroupChunkBytes) {
        const size_t n = table_bytes - off < kGroupChunkBytes ? table_bytes - off : kGroupChunkBytes;
        TableChunk chunk;
        memcpy(chunk.q, src + off, n);
        if (n < kGroupChunkBytes)
            memset(reinterpret_cast<unsigned char *>(chunk.q) + n, 0, kGroupChunkBytes - n);
        hipLaunchKernelGGL(group_table_upload_kernel, dim3(1), dim3(kGroupChunkBytes / 16), 0, stream,
                           reinterpret_cast<uint4 *>(static_cast<unsigned char *>(dev_table) + off), chunk,
                           (int)(n / 16));
        e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    return launch_gemm_group(kind, static_cast<const GroupHeader *>(dev_table), count, workgroups, stream);
}

hipError_t launch_gemm_group(int kind, const GroupHeader *table_dev, uint32_t count, uint32_t workgroups,
                             hipStream_t stream)
{
    // the small-problem instances (first row of each table above): 4 waves x 4 strings by 64 strings per workgroup;
    // the grid is large enough to fill the machine, so the 2-string instances bring nothing here (measured)
    static_assert(kGroupTileS == 4 * 4 && kGroupTileV == 64, "group tile = small-problem instance");
    switch (kind) {
    case KIND_BNN:
        hipLaunchKernelGGL((gemm_group_kernel<KIND_BNN, 4, 1, 4, 16, 8>), dim3(workgroups), dim3(256), 0, stream,
                           table_dev, count);
        break;
    case KIND_TNN:
        hipLaunchKernelGGL((gemm_group_kernel<KIND_TNN, 4, 1, 4, 16, 4>), dim3(workgroups), dim3(256), 0, stream,
                           table_dev, count);
        break;
    case KIND_TBN:
        hipLaunchKernelGGL((gemm_group_kernel<KIND_TBN, 4, 1, 4, 16, 8>), dim3(workgroups), dim3(256), 0, stream,
                           table_dev, count);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gemm_splitk(int kind, const GemmArgs &a, bool transposed, int nsplit)
{
    // 8 x 64 tiles (one string per wave, 8 waves), the instance the selection takes for problems this small
    switch (kind) {
    case KIND_BNN: return launch_splitk<KIND_BNN, 1, 1, 8, 16, 8>(a, transposed, nsplit);
    case KIND_TNN: return launch_splitk<KIND_TNN, 1, 1, 8, 16, 4>(a, transposed, nsplit);
    case KIND_TBN: return launch_splitk<KIND_TBN, 1, 1, 8, 16, 8>(a, transposed, nsplit);
    case KIND_TBN_SV: return launch_splitk<KIND_TBN_SV, 1, 1, 8, 16, 4>(a, transposed, nsplit);
    default: return hipErrorInvalidValue;
    }
}

const GemmVariant *gemm_variants(int kind, int *count)
{
    switch (kind) {
    case KIND_BNN: *count = (int)(sizeof(kBnn) / sizeof(kBnn[0])); return kBnn;
    case KIND_TNN: *count = (int)(sizeof(kTnn) / sizeof(kTnn[0])); return kTnn;
    case KIND_TBN: *count = (int)(sizeof(kTbn) / sizeof(kTbn[0])); return kTbn;
    case KIND_TBN_SV: *count = (int)(sizeof(kTbnSv) / sizeof(kTbnSv[0])); return kTbnSv;
    default: *count = 0; return nullptr;
    }
}

}  // namespace lowbit
