// Ternary x int8 GEMM on the gfx950 int8 matrix cores, fused dequant epilogue.
//
//   acc[m, n] = sum_k q[m, k] * code[n, k]                       (int32, exact)
//   y[m, n]   = (float(acc) * (a_m / 127)) * beta (+ residual)    (fp32, in that order)
//
// Both operands arrive in v_mfma_i32_32x32x32_i8 fragment order, so every load
// is a fully coalesced 1 KB wavefront read and no shuffles are needed:
//   * activations: tiled int8 buffer written by the quantisation kernel,
//   * weights: 2-bit packed blob; a lane's 32-bit word holds its 16 k-values for
//     one MFMA, as offset codes c = code + 1.  Four shift/and pairs expand it to
//     the 16-byte operand.  The MFMA therefore accumulates sum_k q * c, and the
//     epilogue subtracts sum_k q (from the quantisation kernel) to get acc.
// Integer sums are order independent, so the k-order inside a fragment only
// has to agree between the two operands - it does, by construction of the layouts.
// Int8 weights (the higher-precision critic variant) come in the activations' own
// fragment layout and feed the MFMA as they are: no expansion, no offset correction.
//
// Kernels:
//   gemm_lds_kernel    many tokens: both operand tiles of a workgroup (128 tokens
//                      x 128 k, and 256 or 128 weight rows x 128 k still packed)
//                      are staged in LDS with direct global->LDS loads, double
//                      buffered; in GLU mode the epilogue writes
//                      h = max(G,0)^2 U from interleaved gate / up blocks.
//                      A launch of about one tile per compute unit or fewer puts
//                      eight wavefronts of 64 x 32 on the 128 x 128 tile.
//                      gemm_lds_attn_kernel is the wide tile on the q | k | v product of a
//                      uniform batch at head_dim 128: its epilogue rotates q and k and
//                      writes them and v as the fp16 hi / lo fragments the attention
//                      kernel reads (no fp32 rows, no pack kernel).
//                      gemm_lds_w8_kernel is the same loop on int8 weight blobs.
//                      With few tiles and a long k several workgroups share a
//                      tile, each on its own k range (raw int32 partial tiles,
//                      splitk_epilogue_kernel sums and rescales them).
//   gemm_direct_kernel up to a few hundred tokens: no LDS staging, the 4 to 16
//                      wavefronts of a workgroup split k and finish the tile
//                      together through LDS.
// launch_gemm picks among them by how many workgroups each would make.
#include <cstring>

#include "common.hpp"

namespace brl {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr long DIRECT_MAX_WGS = 640;          // 64 x 32 tiles, 8 wavefronts
constexpr long DIRECT16_MAX_WGS = 512;        // 32 x 32 tiles, 16 wavefronts
constexpr long DIRECT16_MAX_WGS_GLU = 900;    // 32 x 32 output tiles of the GLU form, 8 wavefronts
constexpr long NARROW8_MAX_TILES = 320;       // 128 x 128 tiles up to which eight wavefronts share a tile

struct GemmArgs {
    const uint4* A;          // tiled activations, 16 bytes per lane per fragment
    const float* dscale;
    const int32_t* sumq;
    const uint4* wp[3];      // packed weights per segment
    int wfrag;               // uint4 per (32-row block, 128-k super-block) of a weight blob: 64 (2-bit) or 256 (int8)
    const float* beta[3];
    int nb_end[3];
    int n_end[3];
    int nseg;
    int M, nmb, nnb, nsb;
    int tiles_m, tiles_n, group_m;
    float* y;
    int ldy;
    const float* residual;   // [M, ldy] fp32, or bf16 bit patterns when res_bf16 (widened exactly on load)
    int res_bf16;
    int32_t* acc_dbg;
    int fast_epilogue;       // every segment a multiple of 32 rows, ldy % 4 == 0, no debug tap
    double ops;              // int8 operations of the product (for the timing hooks)
    int glu;                 // 1: segments are (gate, up) of equal size, interleaved block by block;
                             //    the epilogue emits h = (max(G,0) * max(G,0)) * U, one column per pair
    int splits;              // > 1: k is cut into `splits` ranges of sb_per_split super-blocks, one workgroup per
    int sb_per_split;        //      (tile, range); raw int32 partial tiles go to `partials` [splits][M][nnb * 32]
    int32_t* partials;       //      and splitk_epilogue_kernel finishes the product
    // attention-operand epilogue (the q | k | v product of a uniform batch, head_dim 128): instead of fp32 rows the
    // kernel writes what the attention kernel reads - q and k rotated (q also scaled) as fp16 hi / lo MFMA fragments,
    // v transposed fragments - see epilogue_attn
    const float* att_cos;    // [S][64]
    const float* att_sin;
    float att_qscale;
    uint4* att_kvf;          // [B][Hkv][NRB][ K: [8][hi,lo] | V: [4][2][hi,lo] ][64 lanes]
    uint4* att_qf;           // [B][Hq][NRB][8][hi,lo][64 lanes]
    int att_S, att_nrb, att_Hq, att_Hkv;
};

// residual element(s) at flat index o (o % 4 == 0 for the four-wide form)
__device__ inline float res_at(const GemmArgs& g, size_t o) {
    if (g.res_bf16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(g.residual)[o] << 16);
    return g.residual[o];
}
__device__ inline float4 res4_at(const GemmArgs& g, size_t o) {
    if (g.res_bf16) {
        const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(g.residual) + o);
        return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                           __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
    }
    return *reinterpret_cast<const float4*>(g.residual + o);
}

__device__ inline v4i expand_codes(uint32_t p) {
    v4i r;
    r.x = (int)(p & 0x03030303u);
    r.y = (int)((p >> 2) & 0x03030303u);
    r.z = (int)((p >> 4) & 0x03030303u);
    r.w = (int)((p >> 6) & 0x03030303u);
    return r;
}

__device__ inline uint32_t pick(const uint4& v, int dd) {
    return dd == 0 ? v.x : dd == 1 ? v.y : dd == 2 ? v.z : v.w;
}

__device__ inline v4i as_v4i(const uint4& u) {
    v4i r;
    r.x = (int)u.x; r.y = (int)u.y; r.z = (int)u.z; r.w = (int)u.w;
    return r;
}

// XCD-aware tile order: workgroup w runs on XCD (w & 7); each XCD gets a
// contiguous run of tiles, walked in groups of `group_m` row tiles so that the
// tiles resident on one XCD share activation and weight panels in its L2.
__device__ inline bool tile_of_block(const GemmArgs& g, int& tile_m, int& tile_n, int& split) {
    const int tiles = g.tiles_m * g.tiles_n;
    const int total = tiles * g.splits;
    const int per_xcd = (total + 7) / 8;
    const int T0 = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || T0 >= total) return false;
    split = T0 / tiles;
    const int T = T0 - split * tiles;
    const int gsz = g.group_m * g.tiles_n;
    const int grp = T / gsz;
    const int first_m = grp * g.group_m;
    const int rows_in_grp = min(g.group_m, g.tiles_m - first_m);
    tile_m = first_m + (T - grp * gsz) % rows_in_grp;
    tile_n = (T - grp * gsz) / rows_in_grp;
    return true;
}

// Segment, first output column and number of valid columns of global weight block gnb.
// In GLU mode block 2 n is gate block n and block 2 n + 1 is up block n; both map to
// output columns 32 n ...
__device__ inline void block_columns(const GemmArgs& g, int gnb, int& seg, int& col0, int& ncols) {
    if (g.glu) {
        seg = gnb & 1;
        col0 = (gnb >> 1) * 32;
        ncols = gnb < g.nnb ? min(32, g.n_end[0] - col0) : 0;
        return;
    }
    int s = 0;
    if (g.nseg > 1 && gnb >= g.nb_end[0]) s = 1;
    if (g.nseg > 2 && gnb >= g.nb_end[1]) s = 2;
    const int nb_begin = s == 0 ? 0 : g.nb_end[s - 1];
    const int n_begin = s == 0 ? 0 : g.n_end[s - 1];
    seg = s;
    col0 = n_begin + (gnb - nb_begin) * 32;
    ncols = gnb < g.nnb ? min(32, g.n_end[s] - col0) : 0;
}

// Where the TN weight blocks of a wavefront live: segment, packed pointer, output columns.
template <int TN>
struct BCols {
    const uint4* ptr[TN];
    int seg[TN], col0[TN], ncols[TN];
    __device__ inline void init(const GemmArgs& g, int nb0, int lane) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int gnb = min(nb0 + j, g.nnb - 1);      // clamped blocks are computed but never stored
            int s, c0, nc;
            block_columns(g, gnb, s, c0, nc);
            const int lnb = g.glu ? (gnb >> 1) : gnb - (s == 0 ? 0 : g.nb_end[s - 1]);
            seg[j] = s;
            col0[j] = c0;
            ncols[j] = (nb0 + j < g.nnb) ? nc : 0;
            ptr[j] = g.wp[s] + (size_t)lnb * g.nsb * g.wfrag + lane;
        }
    }
};

// Epilogue.  In a 32x32 accumulator tile a lane holds column (lane & 31) and rows
// 8*(v/4) + 4*(lane/32) + v%4.  Each half token block of the wavefront (16 rows x
// TN*32 columns; accumulator registers v < 8 or v >= 8) is turned through a
// private LDS region into row-major order, so that the rescale reads 4
// consecutive columns of one row per lane and the result leaves as 16-byte
// stores (512-byte runs per row for TN = 4):
//     y = (float(acc - sum_q[m]) * dscale[m]) * beta[n] (+ residual)
// Tiles whose column blocks are all full take the 16-byte path (token rows past M are
// masked); tiles on the N edge (or with debug taps, or unaligned rows) take a compact
// per-element loop.
template <int TM, int TN>
struct Epi {
    static constexpr int W = TN * 32, LD = W + 4;
    static constexpr int ROWS = TM * 32;          // token rows of a wavefront: (dscale, sum_q) pairs parked after the turn area
    static constexpr int REGION = 16 * LD + 2 * ROWS;   // ints of LDS per wavefront
};

// accumulator registers half*8 .. half*8+7 of the TN tiles of token block i -> row-major 16 x TN*32 ints in scr
template <int TM, int TN>
__device__ inline void scatter_half(v16i (&acc)[TM][TN], int i, int half, int lane, int* scr) {
    constexpr int LD = Epi<TM, TN>::LD;
    const int cl = lane & 31, rh = (lane >> 5) * 4;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 8; ++v) scr[(8 * (v >> 2) + rh + (v & 3)) * LD + j * 32 + cl] = acc[i][j][half * 8 + v];
    __builtin_amdgcn_wave_barrier();
}

// The per-token scale and code sum of the wavefront's rows are fetched once (one row per lane)
// and parked in LDS behind the turn area, so that the passes below wait on LDS only.
template <int TM, int TN>
__device__ inline const int2* park_rows(const GemmArgs& g, int mb0, int lane, int* scr) {
    int2* rows = reinterpret_cast<int2*>(scr + 16 * Epi<TM, TN>::LD);
#pragma unroll
    for (int r = lane; r < TM * 32; r += 64) {
        const int m = min(mb0 * 32 + r, g.M - 1);
        rows[r] = make_int2(__float_as_int(g.dscale[m]), g.sumq ? g.sumq[m] : 0);   // no offset codes: nothing to subtract
    }
    return rows;
}

// h = (max(G,0) * max(G,0)) * U from the gate / up column pairs; 4 columns of one row per lane
template <int TM, int TN>
__device__ inline void epilogue_glu(const GemmArgs& g, v16i (&acc)[TM][TN], int mb0, int nb0, const float (&beta)[TN],
                                    int lane, int* scr) {
    constexpr int LD = Epi<TM, TN>::LD;
    constexpr int LPR = (TN / 2) * 8;            // lanes per row
    constexpr int RPP = 64 / LPR;
    constexpr int NP = 16 / RPP;                 // passes per half token block
    static_assert(64 % LPR == 0, "TN / 2 must be a power of two");
    const int cg = lane % LPR, r0 = lane / LPR;
    const int jj = cg >> 3, cc = 4 * (cg & 7);
    int row[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) row[p] = p * RPP + r0;
    float bg = beta[0], bu = beta[1];
#pragma unroll
    for (int q = 1; q < TN / 2; ++q)
        if (jj == q) { bg = beta[2 * q]; bu = beta[2 * q + 1]; }
    const int col = (nb0 / 2 + jj) * 32 + cc;
    const int2* rows = park_rows<TM, TN>(g, mb0, lane, scr);
#pragma unroll
    for (int idx = 0; idx < 2 * TM; ++idx) {
        const int mbase = (mb0 + (idx >> 1)) * 32 + (idx & 1) * 16;
        scatter_half<TM, TN>(acc, idx >> 1, idx & 1, lane, scr);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int2 rw = rows[idx * 16 + row[p]];
            const float d = __int_as_float(rw.x);
            const int sq = rw.y;
            const int4 ga = *reinterpret_cast<const int4*>(&scr[row[p] * LD + (2 * jj) * 32 + cc]);
            const int4 ua = *reinterpret_cast<const int4*>(&scr[row[p] * LD + (2 * jj + 1) * 32 + cc]);
            const int gi[4] = {ga.x, ga.y, ga.z, ga.w}, ui[4] = {ua.x, ua.y, ua.z, ua.w};
            float hv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float G = ((float)(gi[q] - sq) * d) * bg;
                const float U = ((float)(ui[q] - sq) * d) * bu;
                const float pz = fmaxf(G, 0.f);
                hv[q] = (pz * pz) * U;
            }
            if (mbase + row[p] < g.M)
                *reinterpret_cast<float4*>(g.y + (size_t)(mbase + row[p]) * g.ldy + col) =
                    make_float4(hv[0], hv[1], hv[2], hv[3]);
        }
        __builtin_amdgcn_sched_barrier(0);       // keeps the requests of later half blocks from piling up here
    }
}

// y = (float(acc - sum_q) * dscale) * beta (+ residual); 4 columns of one row per lane
template <int TM, int TN, bool RES>
__device__ inline void epilogue_plain(const GemmArgs& g, v16i (&acc)[TM][TN], int mb0, int nb0,
                                      const float (&beta)[TN], int lane, int* scr) {
    constexpr int LD = Epi<TM, TN>::LD;
    constexpr int LPR = TN * 8;
    constexpr int RPP = 64 / LPR;                // rows per pass (TN a power of two)
    constexpr int NP = 16 / RPP;
    static_assert(64 % LPR == 0, "TN must be a power of two");
    const int c4 = lane % LPR, r0 = lane / LPR;
    int row[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) row[p] = p * RPP + r0;
    float my_beta = beta[0];
#pragma unroll
    for (int j = 1; j < TN; ++j)
        if ((c4 >> 3) == j) my_beta = beta[j];
    const int col = nb0 * 32 + 4 * c4;
    const int2* rows = park_rows<TM, TN>(g, mb0, lane, scr);
#pragma unroll
    for (int idx = 0; idx < 2 * TM; ++idx) {
        const int mbase = (mb0 + (idx >> 1)) * 32 + (idx & 1) * 16;
        // the residual is requested before the LDS turn of this half block and used after it
        constexpr int NPRE = RES ? NP : 1;
        float4 res[NPRE];
        if constexpr (RES) {     // rows past M are clamped for the load and never stored
#pragma unroll
            for (int p = 0; p < NPRE; ++p)
                res[p] = res4_at(g, (size_t)min(mbase + row[p], g.M - 1) * g.ldy + col);
        }
        scatter_half<TM, TN>(acc, idx >> 1, idx & 1, lane, scr);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int2 rw = rows[idx * 16 + row[p]];
            const float d = __int_as_float(rw.x);
            const int sq = rw.y;
            const int4 a = *reinterpret_cast<const int4*>(&scr[row[p] * LD + 4 * c4]);
            float4 val;
            val.x = ((float)(a.x - sq) * d) * my_beta;
            val.y = ((float)(a.y - sq) * d) * my_beta;
            val.z = ((float)(a.z - sq) * d) * my_beta;
            val.w = ((float)(a.w - sq) * d) * my_beta;
            if constexpr (RES) {
                const float4 r = res[p];
                val.x = val.x + r.x; val.y = val.y + r.y; val.z = val.z + r.z; val.w = val.w + r.w;
            }
            if (mbase + row[p] < g.M) *reinterpret_cast<float4*>(g.y + (size_t)(mbase + row[p]) * g.ldy + col) = val;
        }
        __builtin_amdgcn_sched_barrier(0);       // keeps the requests of later half blocks from piling up here
    }
}

template <int TM, int TN>
__device__ inline void epilogue(const GemmArgs& g, v16i (&acc)[TM][TN], int mb0, int nb0, const float (&beta)[TN],
                                int lane, int* scr) {
    constexpr int W = Epi<TM, TN>::W, LD = Epi<TM, TN>::LD;
    // full column blocks take the 16-byte paths (token rows past M are masked there)
    const bool interior = g.fast_epilogue && mb0 * 32 < g.M && nb0 + TN <= g.nnb;
    if (interior) {
        if (g.glu) {
            if constexpr (TN % 2 == 0) epilogue_glu<TM, TN>(g, acc, mb0, nb0, beta, lane, scr);
        } else if (g.residual) {
            epilogue_plain<TM, TN, true>(g, acc, mb0, nb0, beta, lane, scr);
        } else {
            epilogue_plain<TM, TN, false>(g, acc, mb0, nb0, beta, lane, scr);
        }
        return;
    }

    // tiles on the M / N edge, debug taps, unaligned rows: compact per-element loops
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (mb0 + i >= g.nmb) break;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int mbase = (mb0 + i) * 32 + half * 16;
            scatter_half<TM, TN>(acc, i, half, lane, scr);
            if (g.glu) {
#pragma unroll 1
                for (int e = lane; e < 16 * (W / 2); e += 64) {
                    const int row = e / (W / 2), c = e % (W / 2);
                    const int m = mbase + row;
                    const int jj = c >> 5, cc = c & 31;
                    int seg, col0, ncols;
                    block_columns(g, nb0 + 2 * jj, seg, col0, ncols);
                    if (m < g.M && cc < ncols) {
                        const int sq = g.sumq ? g.sumq[m] : 0;
                        const float d = g.dscale[m];
                        const float G = ((float)(scr[row * LD + (2 * jj) * 32 + cc] - sq) * d) * (*g.beta[0]);
                        const float U = ((float)(scr[row * LD + (2 * jj + 1) * 32 + cc] - sq) * d) * (*g.beta[1]);
                        const float pz = fmaxf(G, 0.f);
                        g.y[(size_t)m * g.ldy + col0 + cc] = (pz * pz) * U;
                    }
                }
            } else {
#pragma unroll 1
                for (int e = lane; e < 16 * W; e += 64) {
                    const int row = e / W, c = e % W;
                    const int m = mbase + row;
                    int seg, col0, ncols;
                    block_columns(g, nb0 + (c >> 5), seg, col0, ncols);
                    if (m < g.M && (c & 31) < ncols) {
                        const int a = scr[row * LD + c] - (g.sumq ? g.sumq[m] : 0);
                        const size_t o = (size_t)m * g.ldy + col0 + (c & 31);
                        float val = ((float)a * g.dscale[m]) * (*g.beta[seg]);
                        if (g.residual) val = val + res_at(g, o);
                        g.y[o] = val;
                        if (g.acc_dbg) g.acc_dbg[o] = a;
                    }
                }
            }
        }
    }
}

// Attention operands straight from the q | k | v product (head_dim 128, 32 | S, uniform layout).  A wavefront
// holds two 32-column blocks of one head: columns c .. c + 31 of its first half and the 32 columns 64 further
// on, the rotary partners of the first (the tile loop hands it the weight pieces in that order).  Both blocks
// of a half block of 16 rows are turned through the wavefront's own LDS region; a lane then has eight
// components of a row and their eight partners, rotates both, scales q, splits into fp16 hi / lo and stores
// four whole 16-byte fragment entries.  No other wavefront is involved.  The arithmetic per element is the one
// the separate pack kernel applies to the fp32 rows ((x c -+ x' s) * scale, then hi = fp16, lo = fp16(t - hi))
// on the same fp32 values the plain epilogue would have written, so the fragments hold the same bits.  v needs
// no turn: its transposed fragment order is the accumulator's own lane order.
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// fp32 -> fp16 of a value the compiler must first round to fp32: without the barrier it folds the last multiply
// into the conversion (v_fma_mixlo_f16, one rounding instead of two), and the hi part used for the lo part then
// differs, on ties, from the one that is stored - and from what the pack kernel makes of the fp32 rows in memory
__device__ inline _Float16 half_of_rounded(float x) {
    asm("" : "+v"(x));
    return (_Float16)x;
}

template <int TM, int TN>
__device__ inline void epilogue_attn(const GemmArgs& g, v16i (&acc)[TM][TN], int mb0, int nb0, const float (&beta)[TN],
                                     int lane, int* scr) {
    static_assert(TN == 2, "a block of a head's first half and the block of its rotary partners");
    constexpr int LD = Epi<TM, TN>::LD;
    constexpr int KS = 8, DB = 4, KVFR = KS * 2 + DB * 4;       // 1 KB fragments per key block at head_dim 128
    int seg, col0, ncols;
    block_columns(g, min(nb0, g.nnb - 1), seg, col0, ncols);
    const bool cols_live = nb0 < g.nnb;
    const int head_all = col0 >> 7;                             // head over q | k | v
    const int sub = (col0 >> 5) & 1;                            // which 32 columns of the head's first half
    const float bsel = beta[0];                                 // both blocks lie in one head, i.e. one matrix
    const int2* rows = park_rows<TM, TN>(g, mb0, lane, scr);
    __builtin_amdgcn_wave_barrier();

    if (seg == 2) {
        if (!cols_live) return;
        // v: lane (column dl of block j, h) holds the keys 16 tt + 8 (e >> 2) + 4 h + (e & 3) of step tt
        const int kvh = head_all - g.att_Hq - g.att_Hkv;
        const int dl = lane & 31, h = lane >> 5;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = mb0 + i;
            if (mb >= g.nmb) continue;
            const int b = (mb * 32) / g.att_S, rb = ((mb * 32) % g.att_S) >> 5;
            uint4* dst = g.att_kvf + ((size_t)(b * g.att_Hkv + kvh) * g.att_nrb + rb) * (KVFR * 64);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int r = sub + 2 * j;                      // 32-column block of the head
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    half8 hi, lo;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int v = 8 * tt + e;
                        const int2 rw = rows[i * 32 + 8 * (v >> 2) + 4 * h + (v & 3)];
                        const float y = ((float)(acc[i][j][v] - rw.y) * __int_as_float(rw.x)) * bsel;
                        const _Float16 yh = half_of_rounded(y);
                        hi[e] = yh;
                        lo[e] = (_Float16)(y - (float)yh);
                    }
                    dst[(KS * 2 + (r * 2 + tt) * 2 + 0) * 64 + h * 32 + dl] = __builtin_bit_cast(uint4, hi);
                    dst[(KS * 2 + (r * 2 + tt) * 2 + 1) * 64 + h * 32 + dl] = __builtin_bit_cast(uint4, lo);
                }
            }
        }
        return;
    }
    if (!cols_live) return;

    // q and k: four lanes per row, eight components and their eight partners per lane; one pass per half block
    const int c8 = lane & 3, row = lane >> 2;                     // row of the half block
    const float scale = seg == 0 ? g.att_qscale : 1.0f;
    const int comp = sub * 32 + 8 * c8;                           // first of the lane's components of the first half
    const int ks = comp >> 4, kg = (comp >> 3) & 1;               // the partners are four k-steps on
#pragma unroll
    for (int idx = 0; idx < 2 * TM; ++idx) {
        const int mb = mb0 + (idx >> 1), hb = idx & 1;
        if (mb >= g.nmb) break;
        const int b = (mb * 32) / g.att_S, rb = ((mb * 32) % g.att_S) >> 5;
        // the rotary factors of the lane's row are requested before the turn
        const int pos = rb * 32 + hb * 16 + row;                  // position inside the state
        const float* cp = g.att_cos + (size_t)pos * 64 + comp;
        const float* sp = g.att_sin + (size_t)pos * 64 + comp;
        const float4 c0 = *reinterpret_cast<const float4*>(cp), c1 = *reinterpret_cast<const float4*>(cp + 4);
        const float4 s0 = *reinterpret_cast<const float4*>(sp), s1 = *reinterpret_cast<const float4*>(sp + 4);
        scatter_half<TM, TN>(acc, idx >> 1, hb, lane, scr);
        const int2 rw = rows[idx * 16 + row];
        const float d = __int_as_float(rw.x);
        const int sq = rw.y;
        const int4 a0 = *reinterpret_cast<const int4*>(&scr[row * LD + 8 * c8]);
        const int4 a1 = *reinterpret_cast<const int4*>(&scr[row * LD + 8 * c8 + 4]);
        const int4 p0 = *reinterpret_cast<const int4*>(&scr[row * LD + 32 + 8 * c8]);
        const int4 p1 = *reinterpret_cast<const int4*>(&scr[row * LD + 32 + 8 * c8 + 4]);
        const int ai[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        const int pi[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
        const float cf[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float sf[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        half8 hi1, lo1, hi2, lo2;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float x1 = ((float)(ai[q] - sq) * d) * bsel;    // component of the first half
            const float x2 = ((float)(pi[q] - sq) * d) * bsel;    // its partner, 64 components on
            const float t1 = (x1 * cf[q] - x2 * sf[q]) * scale;
            const float t2 = (x2 * cf[q] + x1 * sf[q]) * scale;
            const _Float16 h1 = half_of_rounded(t1), h2 = half_of_rounded(t2);
            hi1[q] = h1; lo1[q] = (_Float16)(t1 - (float)h1);
            hi2[q] = h2; lo2[q] = (_Float16)(t2 - (float)h2);
        }
        uint4* dst = seg == 0
            ? g.att_qf + ((size_t)(b * g.att_Hq + head_all) * g.att_nrb + rb) * (KS * 2 * 64)
            : g.att_kvf + ((size_t)(b * g.att_Hkv + (head_all - g.att_Hq)) * g.att_nrb + rb) * (KVFR * 64);
        uint4* slot = dst + (ks * 2) * 64 + kg * 32 + hb * 16 + row;
        slot[0] = __builtin_bit_cast(uint4, hi1);
        slot[64] = __builtin_bit_cast(uint4, lo1);               // the lo plane is the next 1 KB fragment
        slot[8 * 64] = __builtin_bit_cast(uint4, hi2);           // four k-steps = eight fragments on
        slot[9 * 64] = __builtin_bit_cast(uint4, lo2);
    }
}

// k-split launches: the raw accumulators of this workgroup's k range, row-major, 16 bytes per lane
template <int TM, int TN>
__device__ inline void epilogue_partial(const GemmArgs& g, v16i (&acc)[TM][TN], int mb0, int nb0, int split, int lane,
                                        int* scr) {
    constexpr int LD = Epi<TM, TN>::LD;
    constexpr int LPR = TN * 8;
    constexpr int RPP = 64 / LPR;
    constexpr int NP = 16 / RPP;
    static_assert(64 % LPR == 0, "TN must be a power of two");
    const int c4 = lane % LPR, r0 = lane / LPR;
    const int ldp = g.nnb * 32;
    const bool col_ok = nb0 + (c4 >> 3) < g.nnb;
    int32_t* dst = g.partials + (size_t)split * g.M * ldp + nb0 * 32 + 4 * c4;
#pragma unroll
    for (int idx = 0; idx < 2 * TM; ++idx) {
        const int mbase = (mb0 + (idx >> 1)) * 32 + (idx & 1) * 16;
        scatter_half<TM, TN>(acc, idx >> 1, idx & 1, lane, scr);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int row = p * RPP + r0;
            const int4 a = *reinterpret_cast<const int4*>(&scr[row * LD + 4 * c4]);
            if (col_ok && mbase + row < g.M) *reinterpret_cast<int4*>(dst + (size_t)(mbase + row) * ldp) = a;
        }
    }
}

// Sums the partial tiles of a k-split launch (exact integer sums) and applies the same rescale as the
// one-pass epilogues.  One thread per token row and four columns of a weight block (a gate / up pair in
// GLU mode).
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(GemmArgs g) {
    const int nob = g.glu ? g.nnb / 2 : g.nnb;                 // output column blocks
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (size_t)g.M * nob * 8) return;
    const int c = 4 * (int)(t & 7), ob = (int)((t >> 3) % nob), m = (int)((t >> 3) / nob);
    const int gnb = g.glu ? 2 * ob : ob;
    int seg, col0, ncols;
    block_columns(g, gnb, seg, col0, ncols);
    if (c >= ncols) return;
    const int ldp = g.nnb * 32;
    int a0[4] = {0, 0, 0, 0}, a1[4] = {0, 0, 0, 0};
    for (int sp = 0; sp < g.splits; ++sp) {
        const int32_t* src = g.partials + ((size_t)sp * g.M + m) * ldp + gnb * 32 + c;
        const int4 v = *reinterpret_cast<const int4*>(src);
        a0[0] += v.x; a0[1] += v.y; a0[2] += v.z; a0[3] += v.w;
        if (g.glu) {
            const int4 u = *reinterpret_cast<const int4*>(src + 32);
            a1[0] += u.x; a1[1] += u.y; a1[2] += u.z; a1[3] += u.w;
        }
    }
    const float d = g.dscale[m];
    const int sq = g.sumq ? g.sumq[m] : 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (c + e >= ncols) break;
        const size_t o = (size_t)m * g.ldy + col0 + c + e;
        if (g.glu) {
            const float G = ((float)(a0[e] - sq) * d) * (*g.beta[0]);
            const float U = ((float)(a1[e] - sq) * d) * (*g.beta[1]);
            const float pz = fmaxf(G, 0.f);
            g.y[o] = (pz * pz) * U;
        } else {
            float val = ((float)(a0[e] - sq) * d) * (*g.beta[seg]);
            if (g.residual) val = val + res_at(g, o);
            g.y[o] = val;
            if (g.acc_dbg) g.acc_dbg[o] = a0[e] - sq;
        }
    }
}

// ---------------------------------------------------------------------------
// Many-token kernel: WM x WN wavefronts, each TM x TN tiles; both operands staged
// through LDS with direct global->LDS loads, double buffered.
// ---------------------------------------------------------------------------
template <int TM, int TN, int WM, int WN, bool W8>
struct LdsTile {
    static constexpr int NW = WM * WN;
    // k-steps (of 32) per stage: a whole super-block for the 2-bit weights; half of one for int8
    // weights, whose stage would otherwise be 32 KB and leave two wavefronts per SIMD
    static constexpr int KD = W8 ? 2 : 4;
    static constexpr int SPB = 4 / KD;                // stages per super-block
    static constexpr int AFR = WM * TM * KD;          // 1 KB activation fragments per stage
    static constexpr int BFR = WN * TN * (W8 ? KD : 1);   // 1 KB pieces of weights per stage: a packed 2-bit block, or
                                                      // the k-step fragments of an int8 block
    static constexpr int STAGE = (AFR + BFR) * 64;    // uint4 elements per stage
    static constexpr int APW = (AFR + NW - 1) / NW, BPW = (BFR + NW - 1) / NW;   // pieces copied per wavefront

    // Request stage t (k-steps t * KD ...) of this wavefront's share: piece c of wavefront w is
    // fragment c*NW + w (lane i's 16 bytes land at offset 16 i).
    static __device__ inline void issue(const uint4* const (&asrc)[APW], const uint4* const (&bsrc)[BPW], int t,
                                        uint4* st, int wave) {
#pragma unroll
        for (int c = 0; c < APW; ++c)
            if (AFR % NW == 0 || c * NW + wave < AFR)
                __builtin_amdgcn_global_load_lds(asrc[c] + (size_t)t * (KD * 64), st + (c * NW + wave) * 64, 16, 0, 0);
#pragma unroll
        for (int c = 0; c < BPW; ++c)
            if (BFR % NW == 0 || c * NW + wave < BFR)
                __builtin_amdgcn_global_load_lds(bsrc[c] + (size_t)t * (W8 ? KD * 64 : 64), st + (AFR + c * NW + wave) * 64,
                                                 16, 0, 0);
    }

    // The MFMAs of one stage.  Activation fragments are requested from LDS two uses before the
    // MFMAs that consume them.
    // p0: the wavefront's first weight piece of the tile; its TN pieces are p0, p0 + PSTR, ...
    template <int PSTR = 1>
    static __device__ inline void compute(v16i (&acc)[TM][TN], const uint4* st, int wm, int p0, int lane) {
        static_assert(PSTR == 1 || !W8, "strided pieces: 2-bit weights only");
        const uint4* sa = st + (wm * TM * KD) * 64 + lane;
        const uint4* sbp = st + (AFR + p0 * (W8 ? KD : 1)) * 64 + lane;
        uint4 bq[W8 ? 1 : TN];
        if constexpr (!W8) {
#pragma unroll
            for (int j = 0; j < TN; ++j) bq[j] = sbp[j * PSTR * 64];
        }
        constexpr int NF = KD * TM;
        uint4 fr[NF];
        fr[0] = sa[0];
        if (NF > 1) fr[1] = sa[(TM > 1 ? KD : 1) * 64];
#pragma unroll
        for (int dd = 0; dd < KD; ++dd) {
            v4i bf[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (W8) bf[j] = as_v4i(sbp[(j * KD + dd) * 64]);
                else bf[j] = expand_codes(pick(bq[j], dd));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int g = dd * TM + i;                       // use index of this fragment
                if (g + 2 < NF) {
                    const int g2 = g + 2, dd2 = g2 / TM, i2 = g2 % TM;
                    fr[g2] = sa[(i2 * KD + dd2) * 64];
                }
                const v4i af = as_v4i(fr[g]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[j], acc[i][j], 0, 0, 0);
            }
        }
    }
};

template <int TM, int TN, int WM, int WN, bool W8, bool ATTN = false>
__device__ __forceinline__ void gemm_lds_body(const GemmArgs& g) {
    using Tile = LdsTile<TM, TN, WM, WN, W8>;
    constexpr int NW = Tile::NW;
    __shared__ __attribute__((aligned(1024))) uint4 stage0[Tile::STAGE];
    __shared__ __attribute__((aligned(1024))) uint4 stage1[Tile::STAGE];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wn = wave % WN, wm = wave / WN;
    int tile_m, tile_n, split;
    if (!tile_of_block(g, tile_m, tile_n, split)) return;

    const int mb_tile0 = tile_m * WM * TM;
    const int mb0 = mb_tile0 + wm * TM;
    const int nb_tile0 = tile_n * WN * TN;
    // weight blocks of the wavefront: TN neighbours, or (attention-operand epilogue) a 32-column block of a head's
    // first half and the block 64 columns on, which holds the rotary partners of its columns
    constexpr int PSTR = ATTN ? 2 : 1;
    const int p0 = ATTN ? (wn >> 1) * 4 + (wn & 1) : wn * TN;
    const int nb0 = nb_tile0 + p0;

    // sources of the stage pieces this wavefront copies (clamped: padding is never stored)
    const uint4* asrc[Tile::APW];
#pragma unroll
    for (int c = 0; c < Tile::APW; ++c) {
        const int f = c * NW + wave;                              // fragment = (token block, k-step of the stage)
        const int mb = min(mb_tile0 + f / Tile::KD, g.nmb - 1);
        asrc[c] = g.A + ((size_t)mb * g.nsb * 4 + f % Tile::KD) * 64 + lane;
    }
    const uint4* bsrc[Tile::BPW];
#pragma unroll
    for (int c = 0; c < Tile::BPW; ++c) {
        const int piece = c * NW + wave;
        BCols<1> one;
        one.init(g, nb_tile0 + (W8 ? piece / Tile::KD : piece), lane);
        bsrc[c] = one.ptr[0] + (W8 ? (piece % Tile::KD) * 64 : 0);
    }

    float beta[TN];
    {
        BCols<TN> bc;
        bc.init(g, nb0, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) beta[j] = *g.beta[bc.seg[j]];
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // Double buffering with two distinct LDS objects: while one is read, the
    // other is filled.  A stage requested in one step is waited for (vmcnt 0)
    // at the top of the next, so its latency hides behind 4*TM*TN MFMAs.
    // stages of this workgroup's k range (one range covering all of k when splits == 1)
    const int sb_first = split * g.sb_per_split * Tile::SPB;
    const int sb_last = min(g.nsb, (split + 1) * g.sb_per_split) * Tile::SPB;
    Tile::issue(asrc, bsrc, sb_first, stage0, wave);
    int sb = sb_first;
    for (; sb + 1 < sb_last; sb += 2) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        Tile::issue(asrc, bsrc, sb + 1, stage1, wave);
        __builtin_amdgcn_sched_barrier(0);       // the copy requests stay ahead of the MFMAs that hide them
        Tile::template compute<PSTR>(acc, stage0, wm, p0, lane);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (sb + 2 < sb_last) Tile::issue(asrc, bsrc, sb + 2, stage0, wave);
        __builtin_amdgcn_sched_barrier(0);
        Tile::template compute<PSTR>(acc, stage1, wm, p0, lane);
    }
    if (sb < sb_last) {
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        Tile::template compute<PSTR>(acc, stage0, wm, p0, lane);
    }

    // the stages are free once every wavefront has left the k loop: reuse them for the epilogue
    __syncthreads();
    static_assert((NW / 2) * Epi<TM, TN>::REGION * 4 <= Tile::STAGE * 16, "half of the epilogue regions per stage");
    int* scr = reinterpret_cast<int*>(wave < NW / 2 ? stage0 : stage1) + (wave % (NW / 2)) * Epi<TM, TN>::REGION;
    if constexpr (ATTN) {
        static_assert(WN == 4 && TN == 2, "a 256-column tile is two heads of 128: four wavefronts of 32 + 32 columns");
        epilogue_attn<TM, TN>(g, acc, mb0, nb0, beta, lane, scr);
    } else if (g.splits > 1) {
        epilogue_partial<TM, TN>(g, acc, mb0, nb0, split, lane, scr);
    } else {
        epilogue<TM, TN>(g, acc, mb0, nb0, beta, lane, scr);
    }
}

template <int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64, 4) void gemm_lds_kernel(GemmArgs g) {
    gemm_lds_body<TM, TN, WM, WN, false>(g);
}

// the wide tile with the attention-operand epilogue (q | k | v product)
__global__ __launch_bounds__(512, 4) void gemm_lds_attn_kernel(GemmArgs g) {
    gemm_lds_body<2, 2, 2, 4, false, true>(g);
}

// the same tile loop on int8 weight blobs
template <int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64, 4) void gemm_lds_w8_kernel(GemmArgs g) {
    gemm_lds_body<TM, TN, WM, WN, true>(g);
}

// ---------------------------------------------------------------------------
// Few-token kernel: operands straight from L2 to registers; WK wavefronts split k.
// ---------------------------------------------------------------------------
template <int TM, int TN, int WM, int WN, int WK, bool W8 = false>
__global__ __launch_bounds__(WM * WN * WK * 64) void gemm_direct_kernel(GemmArgs g) {
    static_assert(WM * WN * WK == 4 || WM * WN * WK == 8 || WM * WN * WK == 16, "4, 8 or 16 wavefronts per workgroup");
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wk = wave % WK;
    const int wn = (wave / WK) % WN;
    const int wm = wave / (WK * WN);
    int tile_m, tile_n, split;
    if (!tile_of_block(g, tile_m, tile_n, split)) return;      // splits == 1 here

    const int mb0 = (tile_m * WM + wm) * TM;
    const int nb0 = (tile_n * WN + wn) * TN;
    const uint4* aptr[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mb = min(mb0 + i, g.nmb - 1);
        aptr[i] = g.A + (size_t)mb * g.nsb * 256 + lane;
    }
    BCols<TN> bc;
    bc.init(g, nb0, lane);
    float beta[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) beta[j] = *g.beta[bc.seg[j]];

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // k-split variants finish the tile with the whole workgroup, one output element per thread and
    // pass; what an element needs from memory (its token's scale and code sum, its residual) is
    // requested here, ahead of the k loop
    constexpr int NT = WM * WN * WK * 64;
    constexpr int EPT = WK > 1 ? (TM * TN * 1024 + NT - 1) / NT : 1;
    float e_d[EPT], e_res[EPT];
    int e_sq[EPT];
    if constexpr (WK > 1) {
        const int ncb = (g.glu && TN > 1) ? TN / 2 : TN;
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int e = threadIdx.x + q * NT;
            const int c = e & 31, jb = (e >> 5) % ncb, r = (e >> 5) / ncb;
            const int m = min(mb0 * 32 + r, g.M - 1);
            int seg, col0, ncols;
            block_columns(g, min(nb0 + (g.glu ? 2 * jb : jb), g.nnb - 1), seg, col0, ncols);
            e_d[q] = g.dscale[m];
            e_sq[q] = g.sumq ? g.sumq[m] : 0;
            e_res[q] = (g.residual && c < ncols) ? res_at(g, (size_t)m * g.ldy + col0 + c) : 0.f;
        }
    }

    const int sb_per = (g.nsb + WK - 1) / WK;
    const int sb_begin = wk * sb_per;
    const int sb_end = min(g.nsb, sb_begin + sb_per);

    if (sb_begin < sb_end) {
        // weights of a super-block per 32-row block: one packed 16-byte piece per lane (2-bit), or the four
        // k-step fragments themselves (int8)
        constexpr int BW = W8 ? 4 : 1;
        uint4 aq[4][TM];
        uint4 bq[BW][TN];
#pragma unroll
        for (int dd = 0; dd < 4; ++dd)
#pragma unroll
            for (int i = 0; i < TM; ++i) aq[dd][i] = aptr[i][((size_t)sb_begin * 4 + dd) * 64];
#pragma unroll
        for (int q = 0; q < BW; ++q)
#pragma unroll
            for (int j = 0; j < TN; ++j) bq[q][j] = bc.ptr[j][((size_t)sb_begin * BW + q) * 64];

        for (int sb = sb_begin; sb < sb_end; ++sb) {
            const int nxt = min(sb + 1, sb_end - 1);
            uint4 bnext[BW][TN];
#pragma unroll
            for (int q = 0; q < BW; ++q)
#pragma unroll
                for (int j = 0; j < TN; ++j) bnext[q][j] = bc.ptr[j][((size_t)nxt * BW + q) * 64];
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) {
                v4i bf[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (W8) bf[j] = as_v4i(bq[dd][j]);
                    else bf[j] = expand_codes(pick(bq[0][j], dd));
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const v4i af = as_v4i(aq[dd][i]);
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[j], acc[i][j], 0, 0, 0);
                }
                // refill this slot with the same k-step of the next super-block
#pragma unroll
                for (int i = 0; i < TM; ++i) aq[dd][i] = aptr[i][((size_t)nxt * 4 + dd) * 64];
            }
#pragma unroll
            for (int q = 0; q < BW; ++q)
#pragma unroll
                for (int j = 0; j < TN; ++j) bq[q][j] = bnext[q][j];
        }
    }

    if constexpr (WK > 1) {
        // k-split: every wavefront parks its partial accumulators in LDS; 32 consecutive threads then
        // take 32 consecutive columns of one token row.  The sum over the k-parts is an exact integer sum.
        static_assert(WM == 1 && WN == 1, "the k-split variants have one tile per workgroup");
        __shared__ int red[WK * TM * TN * 16 * 64];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((wk * TM * TN + i * TN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        __syncthreads();
        const int ncb = (g.glu && TN > 1) ? TN / 2 : TN;                      // output column blocks of the tile
        const int total = TM * 32 * ncb * 32;
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int e = threadIdx.x + q * NT;
            const int c = e & 31, jb = (e >> 5) % ncb, r = (e >> 5) / ncb;     // column, column block, token row of the tile
            const int i = r >> 5, rr = r & 31;
            const int m = mb0 * 32 + r;
            const int v = 4 * (rr >> 3) + (rr & 3), ln = c + 32 * ((rr >> 2) & 1);
            const int j0 = g.glu ? 2 * jb : jb;
            int seg, col0, ncols;
            block_columns(g, min(nb0 + j0, g.nnb - 1), seg, col0, ncols);
            if (e >= total || m >= g.M || nb0 + j0 >= g.nnb || c >= ncols) continue;
            const size_t o = (size_t)m * g.ldy + col0 + c;
            int a0 = 0, a1 = 0;
#pragma unroll
            for (int p = 0; p < WK; ++p) {
                a0 += red[((p * TM * TN + i * TN + j0) * 16 + v) * 64 + ln];
                if (g.glu) a1 += red[((p * TM * TN + i * TN + j0 + 1) * 16 + v) * 64 + ln];
            }
            float bsel = beta[0];
#pragma unroll
            for (int j = 1; j < TN; ++j)
                if (j0 == j) bsel = beta[j];
            if (g.glu) {
                const float G = ((float)(a0 - e_sq[q]) * e_d[q]) * beta[0];
                const float U = ((float)(a1 - e_sq[q]) * e_d[q]) * beta[TN > 1 ? 1 : 0];
                const float pz = fmaxf(G, 0.f);
                g.y[o] = (pz * pz) * U;
            } else {
                float val = ((float)(a0 - e_sq[q]) * e_d[q]) * bsel;
                if (g.residual) val = val + e_res[q];
                g.y[o] = val;
                if (g.acc_dbg) g.acc_dbg[o] = a0 - e_sq[q];
            }
        }
        return;
    }

    __shared__ __attribute__((aligned(16))) int escr[4 * Epi<TM, TN>::REGION];
    epilogue<TM, TN>(g, acc, mb0, nb0, beta, lane, escr + wave * Epi<TM, TN>::REGION);
}

template <int TM, int TN, int WM, int WN, int WK>
int launch_direct(GemmArgs& g, hipStream_t s, bool w8 = false) {
    g.tiles_m = (g.nmb + WM * TM - 1) / (WM * TM);
    g.tiles_n = (g.nnb + WN * TN - 1) / (WN * TN);
    g.group_m = 4;
    const int total = g.tiles_m * g.tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    LaunchTimer tm(BRL_KC_GEMM_NARROW, s, g.ops);
    if (w8)
        hipLaunchKernelGGL((gemm_direct_kernel<TM, TN, WM, WN, WK, true>), dim3(grid), dim3(WM * WN * WK * 64), 0, s, g);
    else
        hipLaunchKernelGGL((gemm_direct_kernel<TM, TN, WM, WN, WK, false>), dim3(grid), dim3(WM * WN * WK * 64), 0, s, g);
    BRL_LAUNCH_CHECK("gemm_direct_kernel");
    return BRL_OK;
}

template <int TM, int TN, int WM, int WN, bool W8>
int launch_lds(GemmArgs& g, hipStream_t s) {
    g.tiles_m = (g.nmb + WM * TM - 1) / (WM * TM);
    g.tiles_n = (g.nnb + WN * TN - 1) / (WN * TN);
    g.group_m = 4;
    const int total = g.tiles_m * g.tiles_n * g.splits;
    const int grid = ((total + 7) / 8) * 8;
    LaunchTimer tm(WN * TN == 8 ? BRL_KC_GEMM : BRL_KC_GEMM_NARROW, s, g.ops);     // 256-column tiles are the wide class
    if constexpr (W8)
        hipLaunchKernelGGL((gemm_lds_w8_kernel<TM, TN, WM, WN>), dim3(grid), dim3(WM * WN * 64), 0, s, g);
    else
        hipLaunchKernelGGL((gemm_lds_kernel<TM, TN, WM, WN>), dim3(grid), dim3(WM * WN * 64), 0, s, g);
    BRL_LAUNCH_CHECK("gemm_lds_kernel");
    if (g.splits > 1) {
        const size_t threads = (size_t)g.M * (g.glu ? g.nnb / 2 : g.nnb) * 8;
        hipLaunchKernelGGL(splitk_epilogue_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, g);
        BRL_LAUNCH_CHECK("splitk_epilogue_kernel");
    }
    return BRL_OK;
}

}  // namespace

namespace {

int device_cus() {
    static const int cus = [] {        // initialised once, thread-safe
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 256;
        }
        return n;
    }();
    return cus;
}

// would launch_gemm run this many-token product on the 128 x 256 tile?  (the rule at the end of launch_gemm)
bool wide_tile_chosen(int nmb, int nnb) {
    const int cus = device_cus();
    const long t_wide = (long)((nmb + 3) / 4) * ((nnb + 7) / 8);
    const long t_narrow = (long)((nmb + 3) / 4) * ((nnb + 3) / 4);
    const double fill_wide = (double)t_wide / (double)(((t_wide + cus - 1) / cus) * cus);
    const double fill_narrow = (double)t_narrow / (double)(((t_narrow + cus - 1) / cus) * cus);
    return t_wide >= 2 * cus && fill_wide >= 0.95 * fill_narrow;
}

}  // namespace

bool gemm_attn_eligible(int M, int n_heads, int n_kv_heads, int head_dim, int S) {
    const int N = (n_heads + 2 * n_kv_heads) * head_dim;
    return head_dim == 128 && S % 32 == 0 && M % 32 == 0 && M % S == 0 && N % 256 == 0 && wide_tile_chosen(M / 32, N / 32);
}

int launch_gemm_attn(const ActBuf& a, const WeightSegs& w, int M, int K, const AttnOperands& out, hipStream_t s) {
    if (w.count != 3 || w.w8 || !gemm_attn_eligible(M, out.n_heads, out.n_kv_heads, 128, out.S) ||
        w.n_end[0] != out.n_heads * 128 || w.n_end[1] - w.n_end[0] != out.n_kv_heads * 128 ||
        w.n_end[2] - w.n_end[1] != out.n_kv_heads * 128) {
        set_error("gemm: the attention-operand epilogue needs the q | k | v product of a uniform batch at head_dim 128");
        return BRL_EINVAL;
    }
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = reinterpret_cast<const uint4*>(a.q);
    g.dscale = a.dscale;
    g.sumq = a.sumq;
    g.wfrag = 64;
    g.nseg = 3;
    for (int i = 0; i < 3; ++i) {
        g.wp[i] = reinterpret_cast<const uint4*>(w.packed[i]);
        g.beta[i] = w.beta[i];
        g.nb_end[i] = w.nb_end[i];
        g.n_end[i] = w.n_end[i];
    }
    g.M = M;
    g.nmb = M / NB;
    g.nnb = w.nb_end[2];
    g.nsb = round_up(K, SBK) / SBK;
    g.ops = 2.0 * (double)M * (double)w.n_end[2] * (double)K;
    g.splits = 1;
    g.sb_per_split = g.nsb;
    g.att_cos = out.cos_t; g.att_sin = out.sin_t; g.att_qscale = out.qscale;
    g.att_kvf = static_cast<uint4*>(out.kvf); g.att_qf = static_cast<uint4*>(out.qf);
    g.att_S = out.S; g.att_nrb = out.S / 32; g.att_Hq = out.n_heads; g.att_Hkv = out.n_kv_heads;
    g.tiles_m = (g.nmb + 3) / 4;
    g.tiles_n = (g.nnb + 7) / 8;
    g.group_m = 4;
    const int total = g.tiles_m * g.tiles_n;
    const int grid = ((total + 7) / 8) * 8;
    LaunchTimer tm(BRL_KC_GEMM_QKV_ATTN, s, g.ops);
    hipLaunchKernelGGL(gemm_lds_attn_kernel, dim3(grid), dim3(512), 0, s, g);
    BRL_LAUNCH_CHECK("gemm_lds_attn_kernel");
    return BRL_OK;
}

int launch_gemm(const ActBuf& a, const WeightSegs& w, int M, int N, int K, float* y, int ldy,
                const float* residual, int32_t* acc_dbg, int glu, hipStream_t s, int res_bf16) {
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = reinterpret_cast<const uint4*>(a.q);
    g.dscale = a.dscale;
    g.sumq = w.w8 ? nullptr : a.sumq;
    g.wfrag = w.w8 ? 256 : 64;
    g.nseg = w.count;
    for (int i = 0; i < 3; ++i) {
        g.wp[i] = reinterpret_cast<const uint4*>(w.packed[i < w.count ? i : 0]);
        g.beta[i] = w.beta[i < w.count ? i : 0];
        g.nb_end[i] = w.nb_end[i < w.count ? i : w.count - 1];
        g.n_end[i] = w.n_end[i < w.count ? i : w.count - 1];
    }
    g.M = M;
    g.nmb = round_up(M, NB) / NB;
    g.nnb = w.nb_end[w.count - 1];
    g.glu = glu;
    if (glu) {
        if (w.count != 2 || w.n_end[1] != 2 * w.n_end[0] || residual || acc_dbg) {
            set_error("gemm: GLU mode needs two equal segments, no residual, no tap");
            return BRL_EINVAL;
        }
        g.nnb = 2 * w.nb_end[0];
    }
    g.nsb = round_up(K, SBK) / SBK;
    g.ops = 2.0 * (double)M * (double)w.n_end[w.count - 1] * (double)K;
    g.y = y;
    g.ldy = ldy;
    g.residual = residual;
    g.res_bf16 = residual ? res_bf16 : 0;
    g.acc_dbg = acc_dbg;
    g.splits = 1;
    g.sb_per_split = g.nsb;
    g.partials = nullptr;
    g.fast_epilogue = (acc_dbg == nullptr && ldy % 4 == 0) ? 1 : 0;
    for (int i = 0; i < w.count; ++i)
        if ((w.n_end[i] - (i ? w.n_end[i - 1] : 0)) % 32 != 0) g.fast_epilogue = 0;
    (void)N;
    // Tile choice: k-split wavefronts for skinny (few-token) problems, where weight
    // streaming bounds the time; LDS-staged big tiles once the grid fills the chip.
    // (up to 16 wavefronts split k for one or two token blocks: the chain of dependent loads per
    // wavefront is what a short state waits for)
    const bool w8 = w.w8 != 0;
    if (glu) {   // a wavefront needs the gate and the up block of a column pair: even TN only
        if (g.nmb <= 1 || (long)g.nmb * (g.nnb / 2) <= DIRECT16_MAX_WGS_GLU) return launch_direct<1, 2, 1, 1, 8>(g, s, w8);
        if (g.nmb <= 2) return launch_direct<2, 2, 1, 1, 4>(g, s, w8);
    } else {
        // Measured at the 2B layer shapes: one 32-row block per workgroup with k over 16 wavefronts wins
        // while that makes at most ~500 workgroups (M <= 128 ... 192); then 64 x 32 tiles with k over 8
        // wavefronts up to ~640 workgroups (M <= ~400 at N = 2560), 1.5 to 3 times faster there than one
        // 128 x 128 tile per compute unit on a fraction of the chip - also with a long k, where they beat
        // the k-split tile launch below.  (The limits were measured with 2-bit weights and are applied to
        // int8 weights as they are.)
        if (g.nmb <= 1 || (long)g.nmb * g.nnb <= DIRECT16_MAX_WGS) return launch_direct<1, 1, 1, 1, 16>(g, s, w8);
        if (g.nmb <= 2 || (long)((g.nmb + 1) / 2) * g.nnb <= DIRECT_MAX_WGS) return launch_direct<2, 1, 1, 1, 8>(g, s, w8);
        if (g.nmb <= 4) return launch_direct<2, 1, 2, 2, 1>(g, s, w8);
    }
    // Few 128 x 128 tiles and a long k (a few hundred tokens, or a narrow output): k is cut so that about
    // two workgroups per compute unit run; the partial tiles go through the scratch area of the
    // activation buffer and a second small kernel.  Integer partial sums: the result is the same.
    {
        const long tiles = (long)((g.nmb + 3) / 4) * ((g.nnb + 3) / 4);
        if (a.splitk && tiles < SPLITK_MAX_TILES) {
            // (measured at the 2B layer shapes, 160 to 1024 tokens: with k = 2560 the second kernel costs more
            //  than the idle compute units, with k = 6912 the cut saves 20 to 30 %)
            int want = (int)((SPLITK_TARGET_WGS + tiles - 1) / tiles);
            const int maxs = g.nsb >= SPLITK_MIN_SB ? g.nsb / 6 : 1;     // long k only, at least 768 k per range
            if (want > maxs) want = maxs;
            if (want >= 2) {
                const int per = (g.nsb + want - 1) / want;
                const int splits = (g.nsb + per - 1) / per;
                if (splits >= 2 && (size_t)splits * M * g.nnb * 32 <= a.splitk_ints) {
                    g.splits = splits;
                    g.sb_per_split = per;
                    g.partials = a.splitk;
                    return w.w8 ? launch_lds<2, 2, 2, 2, true>(g, s) : launch_lds<2, 2, 2, 2, false>(g, s);
                }
            }
        }
    }
    // int8 weights: the LDS-staged 128 x 128 tile (16 KB per stage)
    if (w.w8) return launch_lds<2, 2, 2, 2, true>(g, s);
    // 128 x 256 workgroup tiles (8 wavefronts of 64 x 64, two workgroups per CU) or 128 x 128 tiles
    // (4 wavefronts, four per CU).  The wide tile does about 5 % more work per unit time; the narrow
    // one wins when it spreads the tiles more evenly over the compute units.
    const long t_narrow = (long)((g.nmb + 3) / 4) * ((g.nnb + 3) / 4);
    // About one 128 x 128 tile per compute unit or fewer: the same tile on eight wavefronts of 64 x 32 (two per
    // SIMD from the one resident workgroup instead of one).  Measured at the 2B layer shapes: 640 tokens QKV 21 ->
    // 17 us, O 19 -> 17; 1024 tokens QKV 21 -> 19, O 20 -> 17, down 37 -> 33; 1792 tokens (280 tiles) 4 to 7 %;
    // from 400 tiles on the four-wavefront tile is ahead.  (The GLU epilogue needs column pairs: not for it.)
    if (!glu && t_narrow <= NARROW8_MAX_TILES) return launch_lds<2, 1, 2, 4, false>(g, s);
    if (wide_tile_chosen(g.nmb, g.nnb)) return launch_lds<2, 2, 2, 4, false>(g, s);
    return launch_lds<2, 2, 2, 2, false>(g, s);
}

}  // namespace brl
