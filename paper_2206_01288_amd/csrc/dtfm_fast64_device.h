// Device code shared by the fused kernels of the 64-device shape (N = 64, D_dp = 8, D_pp = 8):
// the matching programme on 16-bit ranks (Eq. 3), Held-Karp in registers (Eq. 4) and the LDS tables.
// Included by dtfm_fast64.hip and dtfm_fast64_allpairs.hip only.
#pragma once

#include "dtfm_internal.h"

#include <math.h>

namespace {


constexpr int NDEV = 64;
// Row stride of the rank table in LDS, in 16-bit entries. 66 instead of 64 skews consecutive rows by
// one 4-byte bank, so that lanes reading the same column of different rows hit different banks.
constexpr int RSTRIDE = 66;
constexpr int BINOM8[9] = {1, 8, 28, 56, 70, 56, 28, 8, 1};
constexpr int BINOM7[8] = {1, 7, 21, 35, 35, 21, 7, 1};

// the subsets of {0..7} grouped by size: LAYER.s[k][i] = i-th subset with k elements, ascending
struct layer_table {
    unsigned char s[9][70];
};
constexpr layer_table make_layers()
{
    layer_table t = {};
    for (int k = 0; k <= 8; k++) {
        int n = 0;
        for (int S = 0; S < 256; S++) {
            int pc = 0;
            for (int b = 0; b < 8; b++) pc += (S >> b) & 1;
            if (pc == k) t.s[k][n++] = (unsigned char)S;
        }
    }
    return t;
}
constexpr layer_table LAYER = make_layers();

// Held-Karp classes: D as a bit mask over {1..7} (bit d set = d in D; bit 0 never set).
// HKC.cls[j][i] = i-th class with j elements (ascending masks), HKC.idx[D] = its index i.
struct hk_class_table {
    unsigned char cls[8][35];
    unsigned char idx[256];
};
constexpr hk_class_table make_hk_classes()
{
    hk_class_table t = {};
    for (int j = 0; j <= 7; j++) {
        int n = 0;
        for (int D = 0; D < 256; D += 2) {
            int pc = 0;
            for (int b = 1; b < 8; b++) pc += (D >> b) & 1;
            if (pc == j) {
                t.cls[j][n] = (unsigned char)D;
                t.idx[D] = (unsigned char)n;
                n++;
            }
        }
    }
    return t;
}
constexpr hk_class_table HKC = make_hk_classes();

// class reached from source class Ds by the relaxation through d (d not in Ds): (Ds xor d) u {d}
constexpr int hk_dest_class(int Ds, int d)
{
    int out = 1 << d;
    for (int e = 1; e < 8; e++)
        if ((Ds >> e) & 1) out |= 1 << (e ^ d);
    return out;
}
// source class of class D through d (d in D): (D \ d) xor d
constexpr int hk_source_class(int D, int d)
{
    int out = 0;
    for (int e = 1; e < 8; e++)
        if (e != d && ((D >> e) & 1)) out |= 1 << (e ^ d);
    return out;
}
// true when, walking the source classes of a layer in ascending index and d ascending within a source,
// (source of D through d) is the first relaxation into D: it initialises D's register instead of
// taking a min. (Two different d can have the same source class, e.g. D = {d, e} through d and e.)
constexpr bool hk_first_into(int D, int d)
{
    const int mine = HKC.idx[hk_source_class(D, d)];
    for (int e = 1; e < 8; e++) {
        if (e == d || !((D >> e) & 1)) continue;
        const int other = HKC.idx[hk_source_class(D, e)];
        if (other < mine || (other == mine && e < d)) return false;
    }
    return true;
}
// The relaxation programme: HKP.step[J][s][d] for source class s of layer J - 1 and d = 1..7:
// 0xFF when d is in the source class (no relaxation), else (index of the destination class in layer
// J) | 0x80 when this relaxation is the first into its destination.
struct hk_program {
    unsigned char step[8][35][8];
};
constexpr hk_program make_hk_program()
{
    hk_program p = {};
    for (int J = 1; J <= 7; J++)
        for (int s = 0; s < BINOM7[J - 1]; s++)
            for (int d = 1; d < 8; d++) {
                const int Ds = HKC.cls[J - 1][s];
                if ((Ds >> d) & 1) {
                    p.step[J][s][d] = 0xFF;
                    continue;
                }
                const int D = hk_dest_class(Ds, d);
                p.step[J][s][d] = (unsigned char)(HKC.idx[D] | (hk_first_into(D, d) ? 0x80 : 0));
            }
    return p;
}
constexpr hk_program HKP = make_hk_program();

// Sharing one candidate's Held-Karp between two groups of 8 lanes. Relabelling the stages by the
// linear map A of Z_2^3 that swaps bits 0 and 1 (offsets 1 <-> 2, 5 <-> 6; 3, 4, 7 fixed) maps a path
// to a path, and offsets to offsets: a second group of lanes whose lane position q stands for stage
// A(q), and whose G[d] holds the edge to stage A(q) xor A(d), runs the same register programme and
// has in the register of class D the entry of class A(D). Each group then only computes the classes
// D <= A(D) (as masks) of every layer, 280 of the 448 relaxations, and gets the others from the
// register of A(D) of the other group (at the lane position A(q)).
constexpr int hk_swap01(int d) { return (d & 4) | ((d & 1) << 1) | ((d >> 1) & 1); }
constexpr int hk_class_image(int D)
{
    int out = 0;
    for (int e = 1; e < 8; e++)
        if ((D >> e) & 1) out |= 1 << hk_swap01(e);
    return out;
}
// HKS.keep[J][i]: class i of layer J is computed by the group itself; HKS.image[J][i]: index of A(class i)
struct hk_split_table {
    bool keep[8][35];
    unsigned char image[8][35];
};
constexpr hk_split_table make_hk_split()
{
    hk_split_table t = {};
    for (int J = 0; J <= 7; J++)
        for (int i = 0; i < BINOM7[J]; i++) {
            const int D = HKC.cls[J][i], AD = hk_class_image(D);
            t.keep[J][i] = D <= AD;
            t.image[J][i] = HKC.idx[AD];
        }
    return t;
}
constexpr hk_split_table HKS = make_hk_split();

// ---- LDS tables shared by a workgroup of the fused kernels ----
constexpr int LDS_RANK_BYTES = ((NDEV * RSTRIDE * 2 + 15) / 16) * 16;   // 8.25 KiB: u16 rank of W_pp
constexpr int LDS_RVAL_BYTES = NDEV * NDEV * 8;                         // 32 KiB: rank -> weight
constexpr int LDS_WDP_BYTES = NDEV * NDEV * 8;                          // 32 KiB: W_dp
constexpr int LDS_TABLES = LDS_RANK_BYTES + LDS_RVAL_BYTES + LDS_WDP_BYTES;
constexpr int WAVES_PER_BLOCK = 8;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a),
                                                                  __builtin_bit_cast(u16x2, b)));
}

// two 16-bit table entries side by side in one register (low half, high half)
__device__ __forceinline__ uint32_t pack2(uint16_t lo, uint16_t hi)
{
    u16x2 v;
    v.x = lo;
    v.y = hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Orders this wavefront's earlier LDS writes before its later LDS reads as seen by other lanes.
// The LDS unit serves one wavefront's requests in order; this only stops the compiler from moving
// accesses across the point.
#define WAVE_LDS_SYNC()                                         \
    do {                                                        \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  \
        __builtin_amdgcn_wave_barrier();                        \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  \
    } while (0)

// ---- lane exchanges inside the 8 lanes of a candidate (data-parallel primitive moves) ----
constexpr int DPP_XOR1 = 0xB1;          // quad permutation [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad permutation [2,3,0,1]
constexpr int DPP_XOR3 = 0x1B;          // quad permutation [3,2,1,0]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i of every 8 takes lane 7 - i: xor 7

template <int CTRL>
__device__ __forceinline__ double dpp_move(double x)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
// value of x at lane (lane xor d), d = 1, 2, 3, 7
__device__ __forceinline__ double lane_xor_direct(double x, int d)
{
    switch (d) {
    case 1: return dpp_move<DPP_XOR1>(x);
    case 2: return dpp_move<DPP_XOR2>(x);
    case 3: return dpp_move<DPP_XOR3>(x);
    default: return dpp_move<DPP_HALF_MIRROR>(x);
    }
}
// the same exchange through the LDS crossbar (no memory access, no vector-ALU slot)
template <int D>
__device__ __forceinline__ double swizzle_xor(double x)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    const int lo = __builtin_amdgcn_ds_swizzle((int)(uint32_t)b, 0x1F | (D << 10));
    const int hi = __builtin_amdgcn_ds_swizzle((int)(uint32_t)(b >> 32), 0x1F | (D << 10));
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
__device__ __forceinline__ double lane_xor_swizzle(double x, int d)
{
    switch (d) {
    case 1: return swizzle_xor<1>(x);
    case 2: return swizzle_xor<2>(x);
    case 3: return swizzle_xor<3>(x);
    case 4: return swizzle_xor<4>(x);
    case 5: return swizzle_xor<5>(x);
    case 6: return swizzle_xor<6>(x);
    default: return swizzle_xor<7>(x);
    }
}
#ifndef HK_SWIZZLE_SET
#define HK_SWIZZLE_SET 0x70   // bit d set: the exchange by d goes through the LDS crossbar
#endif

// One layer of Held-Karp: classes with J elements from the classes with J - 1. Source-major order, so
// that the mirrored copy of a source serves all its relaxations through d = 4, 5, 6. With SPLIT only
// the classes the group keeps (HKS.keep) are computed; the others then come from the other group of
// the candidate through `cross`, the byte address of the lane that holds them (ds_bpermute).
template <int J, bool SPLIT>
__device__ __forceinline__ void hk_layer(const double (&prev)[35], double (&cur)[35], const double (&G)[8], int cross)
{
#pragma unroll
    for (int s = 0; s < BINOM7[J - 1]; s++) {
        const double x = prev[s];
        double xm = 0.0;
        if ((HKP.step[J][s][4] != 0xFF && !((HK_SWIZZLE_SET >> 4) & 1)) ||
            (HKP.step[J][s][5] != 0xFF && !((HK_SWIZZLE_SET >> 5) & 1)) ||
            (HKP.step[J][s][6] != 0xFF && !((HK_SWIZZLE_SET >> 6) & 1)))
            xm = dpp_move<DPP_HALF_MIRROR>(x);
#pragma unroll
        for (int d = 1; d < 8; d++) {
            const int step = HKP.step[J][s][d];
            if (step == 0xFF) continue;
            const int i = step & 0x7F;
            if (SPLIT && !HKS.keep[J][i]) continue;
            // tab[S \ v][u] at u = v xor d, then + Ghat[u][v]
            double moved;
            if ((HK_SWIZZLE_SET >> d) & 1) moved = lane_xor_swizzle(x, d);
            else moved = (d >= 4 && d <= 6) ? lane_xor_direct(xm, d ^ 7) : lane_xor_direct(x, d);
            const double t = __dadd_rn(moved, G[d]);
            cur[i] = (step & 0x80) ? t : fmin(cur[i], t);
        }
    }
    if (SPLIT && J < 7) {
#pragma unroll
        for (int i = 0; i < BINOM7[J]; i++) {
            if (HKS.keep[J][i]) continue;
            const uint64_t b = __builtin_bit_cast(uint64_t, cur[HKS.image[J][i]]);
            const int lo = __builtin_amdgcn_ds_bpermute(cross, (int)(uint32_t)b);
            const int hi = __builtin_amdgcn_ds_bpermute(cross, (int)(uint32_t)(b >> 32));
            cur[i] = __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
        }
    }
}

// Eq. 4 for the candidate of this lane's 8-lane group; G[d] = Ghat[v][v xor d] of the lane's stage v.
// Every lane of the group returns the optimum. With SPLIT the candidate has two groups, lanes l and
// l xor 32; the upper one is relabelled (stage hk_swap01(l & 7), G[d] = Ghat[v][v xor hk_swap01(d)]).
template <bool SPLIT>
__device__ __forceinline__ double hk_registers(const double (&G)[8], int lane)
{
    const int other = lane ^ 32;
    const int cross = 4 * ((other & ~3) | ((other & 1) << 1) | ((other >> 1) & 1));
    double a[35], b[35];
    // one stage: 0; two stages {v, v xor d}: 0 + Ghat
#pragma unroll
    for (int d = 1; d < 8; d++) b[HKC.idx[1 << d]] = G[d];
    hk_layer<2, SPLIT>(b, a, G, cross);
    hk_layer<3, SPLIT>(a, b, G, cross);
    hk_layer<4, SPLIT>(b, a, G, cross);
    hk_layer<5, SPLIT>(a, b, G, cross);
    hk_layer<6, SPLIT>(b, a, G, cross);
    hk_layer<7, SPLIT>(a, b, G, cross);
    double pp = b[0];   // all eight stages, ending in v: min over v
    pp = fmin(pp, dpp_move<DPP_XOR1>(pp));
    pp = fmin(pp, dpp_move<DPP_XOR2>(pp));
    pp = fmin(pp, dpp_move<DPP_HALF_MIRROR>(pp));
    return pp;
}

// byte k (0..7) of a 64-bit value held as two dwords
__device__ __forceinline__ uint32_t byte_of(uint2 v, int k) { return ((k < 4 ? v.x : v.y) >> (8 * (k & 3))) & 0xFFu; }

// index of the stage pair (a, b), a < b, in lexicographic order
__device__ __forceinline__ int pair_index(int a, int b) { return a * 7 - a * (a - 1) / 2 + (b - a - 1); }
// the inverse: e-th pair -> (i, k); the pairs starting with i = 0..6 begin at e = 0, 7, 13, 18, 22, 25, 27
__device__ __forceinline__ void pair8_decode(int e, int &i, int &k)
{
    const int a = (e >= 7) + (e >= 13) + (e >= 18) + (e >= 22) + (e >= 25) + (e >= 27);
    i = a;
    k = e - (a * 7 - a * (a - 1) / 2) + a + 1;
}
// byte k (0..7, not known at compile time) of a 64-bit value held as two dwords
__device__ __forceinline__ uint32_t byte_at(uint2 v, int k) { return ((k < 4 ? v.x : v.y) >> (8 * (k & 3))) & 0xFFu; }

// DataP of one stage (Eq. 2): max over its 8 devices of the row sums, each taken in slot order with
// the device's own slot skipped. W_dp is bitwise symmetric, so the 28 entries above the diagonal serve
// both row sums they appear in; a sum starts from its first term (0.0 + w = w for w >= +0.0).
__device__ __forceinline__ double stage_datap(const double *Wdp, uint2 devs)
{
    uint32_t dv[8];
#pragma unroll
    for (int k = 0; k < 8; k++) dv[k] = byte_of(devs, k);
    double w[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int k = i + 1; k < 8; k++) w[i][k] = w[k][i] = Wdp[dv[i] * NDEV + dv[k]];
    double dp = 0.0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        double sum = 0.0;
        bool first = true;
#pragma unroll
        for (int k = 0; k < 8; k++) {
            if (k == i) continue;
            sum = first ? w[i][k] : __dadd_rn(sum, w[i][k]);
            first = false;
        }
        dp = i == 0 ? sum : fmax(dp, sum);
    }
    return dp;
}

// always true, but not to the compiler: splits straight-line code into basic blocks
__device__ __forceinline__ bool opaque_true()
{
    int t = 1;
    asm volatile("" : "+s"(t));
    return t != 0;
}

// The min-max subset programme of Eq. 3 for two blocks at once (low and high halves of every
// register): after NROWS rows, G[S] for the column subsets S with NROWS elements is the bottleneck
// optimum of matching rows 0 .. NROWS-1 into S. rowdev[h] / coldev[h]: the devices of the rows and of
// the 8 columns of block h, one per byte. With NROWS = 8, G[255] is the optimum of the block; with
// NROWS = 7, G[255 ^ (1 << c)] is the optimum of the 7 rows into all columns but c.
template <int NROWS, bool SPLIT_ROWS>
__device__ __forceinline__ void match_rows(const uint16_t *R, const uint2 (&rowdev)[2], const uint2 (&coldev)[2],
                                           uint32_t (&G)[256])
{
    uint32_t coloff[2][8];
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
        for (int c = 0; c < 8; c++) coloff[h][c] = byte_of(coldev[h], c);
    // rows are gathered one layer ahead of their use; the scheduling barriers keep the
    // register footprint to two rows plus two layers of the table
    uint32_t wnext[8];
    {
        const uint32_t rb0 = byte_of(rowdev[0], 0) * RSTRIDE, rb1 = byte_of(rowdev[1], 0) * RSTRIDE;
#pragma unroll
        for (int c = 0; c < 8; c++) wnext[c] = pack2(R[rb0 + coloff[0][c]], R[rb1 + coloff[1][c]]);
    }
#pragma unroll
    for (int r = 0; r < NROWS; r++) {
        // With SPLIT_ROWS every row from the third on is a basic block of its own (a branch on a value
        // the compiler cannot see, always taken): the instruction scheduler then cannot pile the gathers
        // of all rows, with their LDS bank conflicts, in front of the programme; those of row r + 1 are
        // issued with the arithmetic of row r and hidden behind it. It shortens a lone wavefront's pass
        // by a few per cent; kernels that keep more state alive around the programme do better without.
        if (SPLIT_ROWS && r >= 2 && !opaque_true()) continue;
        // row r of both blocks: w[c] = (rank of block-0 entry (r,c)) | (rank of block-1 entry) << 16
        uint32_t w[8];
#pragma unroll
        for (int c = 0; c < 8; c++) w[c] = wnext[c];
        if (r < NROWS - 1) {
            const uint32_t rb0 = byte_of(rowdev[0], r + 1) * RSTRIDE, rb1 = byte_of(rowdev[1], r + 1) * RSTRIDE;
#pragma unroll
            for (int c = 0; c < 8; c++) wnext[c] = pack2(R[rb0 + coloff[0][c]], R[rb1 + coloff[1][c]]);
        }
#pragma unroll
        for (int i = 0; i < BINOM8[r + 1]; i++) {
            const int S = LAYER.s[r + 1][i];
            uint32_t acc = 0;
            bool first = true;
#pragma unroll
            for (int c = 0; c < 8; c++) {
                if (!(S & (1 << c))) continue;
                const uint32_t m = (r == 0) ? w[c] : pk_max(G[S ^ (1 << c)], w[c]);
                acc = first ? m : pk_min(acc, m);
                first = false;
            }
            G[S] = acc;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Copies the rank table (rows re-strided), the rank values and W_dp into the workgroup's LDS; the
// caller ends the set-up with a workgroup barrier. EAGER unrolls the copy loops so that a thread's
// loads are all in flight before its first LDS write waits for one: worth 0.5 us of a launch's 3 us
// set-up where that matters (small populations); the long-running kernels keep the plain loops.
template <bool EAGER>
__device__ __forceinline__ void stage_tables(unsigned char *smem, const uint16_t *rank_tab, const double *rank_val,
                                             const double *W_dp)
{
    if (EAGER) {
#pragma unroll 8
        for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
            const int row = i / (NDEV / 2), col2 = i - row * (NDEV / 2);
            reinterpret_cast<uint32_t *>(smem)[row * (RSTRIDE / 2) + col2] = reinterpret_cast<const uint32_t *>(rank_tab)[i];
        }
#pragma unroll 8
        for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
            reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES)[i] = reinterpret_cast<const double2 *>(rank_val)[i];
            reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES)[i] = reinterpret_cast<const double2 *>(W_dp)[i];
        }
    } else {
        for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
            const int row = i / (NDEV / 2), col2 = i - row * (NDEV / 2);
            reinterpret_cast<uint32_t *>(smem)[row * (RSTRIDE / 2) + col2] = reinterpret_cast<const uint32_t *>(rank_tab)[i];
        }
        for (int i = threadIdx.x; i < NDEV * NDEV / 2; i += blockDim.x) {
            reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES)[i] = reinterpret_cast<const double2 *>(rank_val)[i];
            reinterpret_cast<double2 *>(smem + LDS_RANK_BYTES + LDS_RVAL_BYTES)[i] = reinterpret_cast<const double2 *>(W_dp)[i];
        }
    }
}

}  // namespace
