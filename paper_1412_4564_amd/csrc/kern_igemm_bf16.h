// Implicit-GEMM convolution on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16):
// the "operands rounded to bf16 on chip, fp32 accumulation" variant of kern_igemm.h.
// Arrays in memory stay fp32 in the layout of the MatConvNet manual (arXiv 1412.4564,
// Sec. 2.3.1); the sum computed is the one of Sec. 4.1 (see kern_igemm.h), with every x and
// w rounded to bf16 (round to nearest even) before the products are formed.
//
// Same tiling, same pixel numbering, same stream-K scheduling, same fix-up pass and the same
// IgemmParams as the fp32 kernel.  What differs:
//  * one MFMA consumes 16 reduction elements: 16 channels of one filter tap.  Lane l holds
//    8 consecutive channels (octet l/32 of the 16) of filter or pixel l%32, as one 16-byte
//    register group, so both operands are stored channel-interleaved:
//      slab     [octet][column][row][8 channels]  bf16, 16 bytes per (octet, sample)
//      weights  [step][octet][filter][8 channels] bf16 (written that way by the packing pass)
//    and every operand read is one ds_read_b128 of consecutive 16-byte words (conflict-free).
//    P.CP is the slab's pitch per octet in samples, P.DC = 16, a step is one tap (P.NS = P.TC),
//    P.WSZ counts 32-bit words of packed weights per unit.
//  * the slab cannot be loaded straight into LDS: a thread loads the 16 channels of its
//    sample(s) into registers one unit ahead (coalesced along rows, as before), and after
//    the unit's MFMAs converts them and writes two 16-byte words.
//  * a unit is 16 channels x one range of taps; the slab depends on the channels only, so it is
//    staged when a unit starts a new group of 16 channels (or the block's range) and kept for the
//    units of the group's other tap ranges.
//
// Split operands (template parameter PL = 2, "bf16x3"): every fp32 value v is held as two bf16 planes,
// hi = bf16(v) and lo = bf16(v - hi), which together carry 16 bits of its significand, and every product
// w*x is formed as  w_hi*x_hi + w_hi*x_lo + w_lo*x_hi  (three MFMAs; the dropped w_lo*x_lo is below 2^-16 of
// |w||x|, the two roundings to lo below 2^-17 each).  The sum is that of Sec. 4.1 with products exact to
// about 1e-5 of |w||x| in the worst case, on a matrix core that runs these MFMAs 16 times as fast as the
// fp32 ones.  Planes sit side by side: slab [plane][octet][sample][8], weights [step][plane][octet][filter][8].
#pragma once
#include "kern_igemm.h"

namespace mcn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int BF_DC = 16;        // channels per unit = reduction depth of one MFMA
// slab samples a thread stages per unit, at most (16 registers each)
constexpr int bf_ept_max(int threads) { return threads <= 256 ? 4 : 2; }

__device__ inline unsigned pack_bf16x2(float lo, float hi) {
    const floatx2 v = {lo, hi};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);     // round to nearest even
    return __builtin_bit_cast(unsigned, h);
}

// hi and lo planes of a pair of fp32 values: hi = bf16(v), lo = bf16(v - hi) (the difference is exact in fp32)
__device__ inline void split_bf16x2(float v0, float v1, unsigned *hi, unsigned *lo) {
    const unsigned h = pack_bf16x2(v0, v1);
    *hi = h;
    *lo = pack_bf16x2(v0 - __uint_as_float(h << 16), v1 - __uint_as_float(h & 0xffff0000u));
}

// packed[g][kt][unit][step][plane][octet][kk][8 channels] as bf16 (Q.planes = 1: the values rounded to bf16;
// 2: their hi and lo planes); one thread writes one pair of channels (a 32-bit word).  Modes as in
// igemm_pack_weights_kernel.
__global__ __launch_bounds__(256) void igemm_pack_weights_bf16_kernel(const float *__restrict__ w,
                                                                      unsigned *__restrict__ packed, PackParams Q) {
    int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= Q.total) return;
    int t = p / Q.WSZ;
    int within = p - t * Q.WSZ;
    const int j2 = within & 3; within >>= 2;
    const int kk = within % Q.TK; within /= Q.TK;
    const int oct = within & 1; within >>= 1;
    const int plane = within % Q.planes;
    const int s = within / Q.planes;             // tap of the unit's tap range
    const int uu = t % Q.NU; t /= Q.NU;
    const int kt = t % Q.KT;
    const int g = t / Q.KT;
    const int cg = uu / Q.NTR, tr = uu - cg * Q.NTR;
    const int tap = tr * Q.TC + s;
    const int k = kt * Q.TK + kk;
    float v[2] = {0.f, 0.f};
    if (s < Q.TC && tap < Q.Hf * Q.Wf && k < Q.Kg) {
        const int ti = tap % Q.Hf, tj = tap / Q.Hf;
        for (int e = 0; e < 2; ++e) {
            const int c = cg * BF_DC + oct * 8 + 2 * j2 + e;
            if (c >= Q.Cg) continue;
            if (Q.mode == 0) {
                v[e] = w[ti + Q.HfA * (tj + Q.WfA * (c + (size_t)Q.DfA * (g * Q.Kg + k)))];
            } else if (Q.mode == 1) {
                const int fi = Q.pi + Q.Sh * (Q.Hf - 1 - ti), fj = Q.pj + Q.Sw * (Q.Wf - 1 - tj);
                v[e] = w[fi + Q.HfA * (fj + Q.WfA * (k + (size_t)Q.DfA * (g * Q.Cg + c)))];
            } else {
                v[e] = w[k + (size_t)Q.ldk * c];
            }
        }
    }
    unsigned hi, lo;
    split_bf16x2(v[0], v[1], &hi, &lo);
    packed[p] = plane ? lo : hi;
}

// WK x WP waves; each wave owns MK x MP tiles of 32 filters x 32 pixels.
// LW more waves stage the operands (load, convert, write the slab; the packed weights go
// straight to LDS) while the WK x WP waves only read LDS and issue MFMAs; see igemm_sk_kernel.
// PL: operand planes (1: values rounded to bf16; 2: hi and lo planes, three products per pair of operands)
template <int WK, int WP, int MK, int MP, int WPE, int LW, int PL = 1>
__global__ __launch_bounds__(64 * (WK * WP + LW), WPE) void igemm_bf16_kernel(IgemmParams P, const float *__restrict__ in,
                                                                       const float *__restrict__ wpk,
                                                                       const float *__restrict__ bias,
                                                                       float *__restrict__ out,
                                                                       float *__restrict__ part) {
    constexpr int NT = 64 * WK * WP;               // computing threads
    static_assert(LW > 0, "the computing waves do not stage operands");
    constexpr int NL = 64 * LW;                    // staging threads
    constexpr int NLW = LW;                        // staging waves
    constexpr int TK = WK * MK * 32;
    constexpr int TQ = WP * MP * 32;
    constexpr int BF_EPT_MAX = bf_ept_max(NL);
    static_assert(NLW * 64 >= TK, "the staging waves fetch one bias value per lane");
    const int NS = P.NS;
    const int NU = P.NU;
    const int WSZ = P.WSZ;               // 32-bit words of packed weights per unit
    const int CP = P.CP, SRP = P.SRP;
    const int XSZ = PL * 2 * CP * 4;     // 32-bit words of slab per buffer: PL planes x 2 octets x CP samples x 16 bytes

    extern __shared__ __align__(16) float lds[];
    float *wbuf = lds;                                   // [2][WSZ]
    float *xbuf = lds + 2 * WSZ;                         // [2][XSZ]
    int *gtab = reinterpret_cast<int *>(xbuf + 2 * XSZ); // [EPT][NL]: entry (s, t) is private to staging thread t
    float *blds = reinterpret_cast<float *>(gtab + P.EPT * NL);   // [2][TK] bias of the tile, slots used in turn

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wp = (wave / WK) % WP;
    const bool loader = wave >= WK * WP;                    // whole waves
    const int ltid = tid - NT;                              // index among the staging threads
    const int lwave = wave - WK * WP;
    const int HW = P.H * P.W;
    const int OHW = P.OH * P.OW;

    const int vb = sk_virtual_block(blockIdx.x, P.nblocks);
    const int tile_s0 = P.own * P.nblocks;                          // first shared tile
    const long long total = (long long)(P.tiles - tile_s0) * NU;    // units of the shared tiles
    const int rank = sk_share_rank(P.nblocks, P.nshare, vb);
    const long long ub = rank < 0 ? 0 : sk_begin(total, P.nshare, rank), ue = rank < 0 ? 0 : sk_begin(total, P.nshare, rank + 1);
    const int n_own = P.own * NU;                                    // units of this block's own tiles
    const int nunits = n_own + (int)(ue - ub);
    if (nunits == 0) return;

    const buffer_rsrc wrs = make_rsrc(wpk, P.packed_bytes);
    const buffer_rsrc brs = make_rsrc(bias, bias ? (unsigned)P.Ktot * 4u : 0u);
    const unsigned lane16 = (unsigned)lane * 16u;

    // ---- load side: tile whose units are being fetched ------------------------------------
    __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void *)in, 0, 0, BUFFER_FLAGS);
    unsigned wtile_off = 0;        // byte offset of the tile's packed weights
    int l_kt = 0, l_g = 0;
    int l_seq = -1, c_seq = -1;    // how many tiles the load / the compute side has started: picks the bias slot
    auto setup_load = [&](int t) {
        ++l_seq;
        int kt, pt, rb, g;
        decode_tile(P, t, &kt, &pt, &rb, &g);
        const int q0 = pt * TQ;
        const int c_first = div32(q0, P.dTI);
        const int n_first = div32(c_first, P.dWo);
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;   // chained column of the slab's first column
        const int row0 = rb * P.TI * P.Sh - P.Pt;           // input row of slab row 0
        const size_t in_base = ((size_t)n_first * P.Ctot + (size_t)g * P.Cg) * HW;
        size_t in_left = ((size_t)P.N * P.Ctot * HW - in_base) * 4;
        if (in_left > 0x7fffffffull) in_left = 0x7fffffffull;
        xrs = __builtin_amdgcn_make_buffer_rsrc((void *)(in + in_base), 0, (int)in_left, BUFFER_FLAGS);
        wtile_off = (unsigned)((size_t)(g * P.KT + kt) * NU * WSZ * 4);
        l_kt = kt; l_g = g;
        for (int s = 0; s < P.EPT; ++s) {
            const int e = ltid + NL * s;
            const int col = div32(e, P.dSRP);
            const int r = e - col * SRP;
            const int U = u0 + col;
            const int ni = div32(U, P.dWp);          // image relative to n_first
            const int j = U - ni * P.Wp - P.Pl;
            const int i = row0 + r;
            const bool ok = e < CP && r < P.SR && i >= 0 && i < P.H && j >= 0 && j < P.W && (n_first + ni) < P.N;
            gtab[s * NL + ltid] = ok ? (int)(4u * (unsigned)(i + P.H * j + ni * P.Ctot * HW)) : (int)SLAB_INVALID;
        }
    };
    // the 16 channels of this thread's slab samples, held in registers while the unit before is computed
    float stg[BF_EPT_MAX][BF_DC];
    // weights (and bias) of unit uu into weight buffer b; with_slab: the unit starts a group of channels (or the
    // block's range), so the group's samples are fetched into registers as well
    auto issue_loads = [&](int uu, int b, bool with_slab) {
        float *wb = wbuf + b * WSZ;
        const unsigned woff = wtile_off + (unsigned)uu * (unsigned)WSZ * 4u;
        for (int e0 = lwave * 256; e0 < WSZ; e0 += NLW * 256)     // one wave instruction = 1 KB, 16 bytes per lane
            load_to_lds_b128(lds_address(wb + e0), lane16, wrs, woff + (unsigned)e0 * 4u);
        if (bias && uu == 0 && lwave * 64 < TK) {
            // the tile's bias: start value of the accumulators of a tile this block owns entirely
            const int kl = l_kt * TK + lwave * 64 + lane;
            if (lwave * 64 + lane < TK)
                load_to_lds_b32(lds_address(blds + (l_seq & 1) * TK + lwave * 64),
                                kl < P.Kg ? (unsigned)(l_g * P.Kg + kl) * 4u : SLAB_INVALID, brs, 0);
        }
        if (!with_slab) return;
        const int c0 = (P.NTR == 1 ? uu : uu / P.NTR) * BF_DC;      // one tap range is the common case: no division
        const bool full = c0 + BF_DC <= P.Cg;
#pragma unroll
        for (int s = 0; s < BF_EPT_MAX; ++s) {
            if (s < P.EPT && lwave * 64 + NL * s < CP) {
                const unsigned go = (unsigned)gtab[s * NL + ltid];
                if (full) {
#pragma unroll
                    for (int d = 0; d < BF_DC; ++d)
                        stg[s][d] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                            xrs, go, (unsigned)(c0 + d) * (unsigned)HW * 4u, 0));
                } else {
#pragma unroll
                    for (int d = 0; d < BF_DC; ++d) {
                        const int c = c0 + d;
                        // channels past the group's last one read as zero (their weights are zero too)
                        stg[s][d] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                            xrs, c < P.Cg ? go : SLAB_INVALID, (unsigned)c * (unsigned)HW * 4u, 0));
                    }
                }
            }
        }
    };
    // convert the staged samples and publish them in slab buffer b
    auto write_slab = [&](int b) {
        float *xb = xbuf + b * XSZ;
#pragma unroll
        for (int s = 0; s < BF_EPT_MAX; ++s) {
            if (s < P.EPT && lwave * 64 + NL * s < CP) {
                const int e = ltid + NL * s;
#pragma unroll
                for (int o = 0; o < 2; ++o) {
                    unsigned hi[4], lo[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) split_bf16x2(stg[s][8 * o + 2 * j], stg[s][8 * o + 2 * j + 1], &hi[j], &lo[j]);
                    const uintx4 v = {hi[0], hi[1], hi[2], hi[3]}, l = {lo[0], lo[1], lo[2], lo[3]};
                    *reinterpret_cast<uintx4 *>(xb + (size_t)(o * CP + e) * 4) = v;
                    if constexpr (PL == 2) *reinterpret_cast<uintx4 *>(xb + (size_t)((2 + o) * CP + e) * 4) = l;
                }
            }
        }
    };

    // ---- compute side: tile whose accumulators are live -----------------------------------
    int bbase[MP];       // slab byte offset of the pixel's window origin, octet of this half-wave
    unsigned ooff[MP];   // byte offset of the lane's first result of the tile relative to the tile's output
                         // window (filter k0 + 4*half of image n_first), or SLAB_INVALID
    __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc((void *)out, 0, 0, BUFFER_FLAGS);   // the tile's output window
    int c_kt = 0, c_g = 0;
    bool need_init = true;
    floatx16 acc[MK][MP];
    auto setup_compute = [&](int t) {
        ++c_seq;
        int kt, pt, rb, g;
        decode_tile(P, t, &kt, &pt, &rb, &g);
        c_kt = kt; c_g = g;
        const int q0 = pt * TQ;
        const int qend = min(q0 + TQ, P.QN);
        const int c_first = div32(q0, P.dTI);
        const int n_first = div32(c_first, P.dWo);
        const int u0 = (c_first - n_first * P.Wo) * P.Sw;
#pragma unroll
        for (int mp = 0; mp < MP; ++mp) {
            const int q = q0 + (wp * MP + mp) * 32 + (lane & 31);
            const int c = div32(q, P.dTI);
            const int ii = q - c * P.TI;
            const int n = div32(c, P.dWo);
            const int jo = c - n * P.Wo;
            const int io = rb * P.TI + ii;
            const bool ok = q < qend && io < P.Ho;
            const int ucol = jo * P.Sw + (n - n_first) * P.Wp - u0;
            bbase[mp] = 16 * ((ok ? ii * P.Sh + SRP * ucol : 0) + half * CP);
            ooff[mp] = ok ? 4u * (unsigned)((P.oi0 + P.osi * io) + P.OH * (P.oj0 + P.osj * jo) +
                                            OHW * (P.Ktot * (n - n_first) + 4 * half))
                          : SLAB_INVALID;
        }
        const size_t out_base = (size_t)n_first * P.Ktot * OHW;
        size_t out_left = ((size_t)P.N * P.Ktot * OHW - out_base) * 4;
        if (out_left > 0x7fffffffull) out_left = 0x7fffffffull;
        ors = __builtin_amdgcn_make_buffer_rsrc((void *)(out + out_base), 0, (int)out_left, BUFFER_FLAGS);
        need_init = true;
    };
    auto init_acc = [&](bool with_bias) {
        const float *bl = blds + (c_seq & 1) * TK;
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                const float bv = with_bias ? bl[kloc] : 0.f;
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) acc[mk][mp][v] = bv;
            }
    };
    const int aoff = 16 * (half * TK + wk * MK * 32 + (lane & 31));   // bytes
    // One step per tap of the unit's tap range.  The slab offset of the tap is kept in scalar registers
    // (fi, fj run along; a step past the filter's last tap has zero weights and reads offset 0), the
    // operands of step s+1 are requested before the MFMAs of step s, and the loop body has no branches
    // so that the waits inserted for the LDS reads are exact.
    auto compute = [&](int uu, int b, int xb) {
        const char *wl = reinterpret_cast<const char *>(wbuf + b * WSZ) + aoff;
        const char *xl = reinterpret_cast<const char *>(xbuf + xb * XSZ);
        const int T = P.Hf * P.Wf;
        int tap = 0, fj = 0, fi = 0;
        if (P.NTR != 1) {
            tap = (uu % P.NTR) * P.TC;
            fj = tap / P.Hf;
            fi = tap - fj * P.Hf;
        }
        int so = 16 * (fj * SRP + fi);                   // byte offset of the current tap in the slab
        // operand registers: [plane * M + m]
        bf16x8 a0[PL * MK], b0[PL * MP], a1[PL * MK], b1[PL * MP];
        const int xplane = 2 * CP * 16;                  // bytes from a slab plane to the next
        auto fetch = [&](bf16x8 *a, bf16x8 *bq) {
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) {
#pragma unroll
                for (int mk = 0; mk < MK; ++mk) a[pl * MK + mk] = *reinterpret_cast<const bf16x8 *>(wl + (pl * 2 * TK + mk * 32) * 16);
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) bq[pl * MP + mp] = *reinterpret_cast<const bf16x8 *>(xl + bbase[mp] + so + pl * xplane);
            }
            wl += PL * 2 * TK * 16;
            // next tap (all scalar)
            ++tap;
            const bool wrap = ++fi == P.Hf;
            so += wrap ? 16 * (SRP - P.Hf + 1) : 16;
            if (wrap) fi = 0;
            if (tap >= T) so = 0;
        };
        auto mma = [&](const bf16x8 *a, const bf16x8 *bq) {
            if constexpr (PL == 2) {
                // the two small products first, then the large one
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp)
                        acc[mk][mp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[MK + mk], bq[mp], acc[mk][mp], 0, 0, 0);
#pragma unroll
                for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                    for (int mp = 0; mp < MP; ++mp)
                        acc[mk][mp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mk], bq[MP + mp], acc[mk][mp], 0, 0, 0);
            }
#pragma unroll
            for (int mk = 0; mk < MK; ++mk)
#pragma unroll
                for (int mp = 0; mp < MP; ++mp)
                    acc[mk][mp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mk], bq[mp], acc[mk][mp], 0, 0, 0);
        };
        fetch(a0, b0);
        for (int s = 2; s < NS; s += 2) {        // steps s-2 and s-1, with s-1 and s in flight
            fetch(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            fetch(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mma(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (NS & 1) {
            mma(a0, b0);
        } else {
            fetch(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mma(a0, b0);
            mma(a1, b1);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int mk = 0; mk < MK; ++mk) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kl0 = c_kt * TK + (wk * MK + mk) * 32 + (v >> 2) * 8 + (v & 3);   // filter of the lower half-wave
                const int left = P.Kg - kl0;
                if (left <= 0) continue;
                const unsigned soff = (unsigned)(c_g * P.Kg + kl0) * (unsigned)OHW * 4u;
#pragma unroll
                for (int mp = 0; mp < MP; ++mp) {
                    const unsigned vo = (left > 4 || half == 0) ? ooff[mp] : SLAB_INVALID;   // the upper half-wave holds filter kl0 + 4
                    float val = acc[mk][mp][v];
                    if (P.relu) val = fmaxf(val, 0.f);
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), ors, vo, soff, 0);
                }
            }
        }
    };
    auto store_partial = [&](int slot) {
        float *dst = part + (size_t)slot * (TK * TQ);
#pragma unroll
        for (int mk = 0; mk < MK; ++mk)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kloc = (wk * MK + mk) * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
#pragma unroll
                for (int mp = 0; mp < MP; ++mp)
                    dst[kloc * TQ + (wp * MP + mp) * 32 + (lane & 31)] = acc[mk][mp][v];
            }
    };

    // ---- the block's range of units --------------------------------------------------------
    // position = (tile, unit); `done` = units consumed so far.  After the block's own tiles comes its range
    // of the shared ones, which may start in the middle of a tile.
    const int t_s = tile_s0 + (int)(ub / NU), uu_s = (int)(ub - (ub / NU) * NU);
    // returns whether the next unit starts a new slab: a new group of channels, a new tile, or the jump from the
    // block's own tiles to its range of the shared ones (which may land inside a group)
    auto advance = [&](int &t, int &uu, int done) {
        if (done == n_own) { t = t_s; uu = uu_s; return true; }
        if (++uu == NU) { uu = 0; ++t; }
        return P.NTR == 1 || uu % P.NTR == 0;
    };
    // the whole tiles of a block, dealt among the blocks of its XCD as in igemm_sk_kernel (neighbouring tiles are
    // then in flight on one XCD together and share its L2)
    auto tile_of = [&](int t) {
        if (t >= tile_s0 || (P.nblocks & 7) != 0) return t;
        const int b = t / P.own, j = t - b * P.own;
        const int G = P.nblocks >> 3, x = b / G, i = b - x * G;
        return (x * G) * P.own + j * G + i;
    };
    int t_c = n_own ? vb * P.own : t_s;   // compute-side tile and unit
    int uu_c = n_own ? 0 : uu_s;
    int t_l = t_c, uu_l = uu_c;           // the load side runs one unit ahead
    bool first_segment = true;
    // the segment starting at unit uu of tile t covers the tile iff the tile is the block's own, or it
    // starts at 0 and the block's shared range reaches the tile's end
    auto segment_is_whole = [&](int t, int uu) {
        return t < tile_s0 || (uu == 0 && (long long)(t - tile_s0 + 1) * NU <= ue);
    };
    if (loader) {
        // Staging wave: unit it+1 goes into the buffers the computing waves left at the barrier of
        // iteration it, and is complete (weights landed, slab written) before the next barrier.
        // Slab buffers are used in turn, one per group of channels: the buffer written for the next group was last
        // read by the group before the current one, whose units ended at an earlier barrier.
        int slab = 0;
        setup_load(tile_of(t_l));
        issue_loads(uu_l, 0, true);
        write_slab(0);
        for (int it = 0; it < nunits; ++it) {
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
            lds_barrier();
            if (it + 1 < nunits) {
                const int t_prev = t_l;
                const bool fresh = advance(t_l, uu_l, it + 1);
                if (t_l != t_prev) setup_load(tile_of(t_l));
                issue_loads(uu_l, (it + 1) & 1, fresh);
                if (fresh) { slab ^= 1; write_slab(slab); }
            }
        }
        return;
    }
    bool whole = segment_is_whole(t_c, uu_c);
    setup_compute(tile_of(t_c));

    int slab_c = 0;                                // slab buffer of the current unit (see the staging waves)
    for (int it = 0; it < nunits; ++it) {
        lds_barrier();                             // the staging waves' operands are in place, and the other buffer is free
        if (need_init) { init_acc(whole && bias != nullptr); need_init = false; }
        __builtin_amdgcn_sched_barrier(0);
        compute(uu_c, it & 1, slab_c);
        __builtin_amdgcn_sched_barrier(0);
        const bool last = it + 1 == nunits;
        if (uu_c + 1 == NU || last) {
            if (whole) store_tile();
            else store_partial(2 * vb + (first_segment ? 0 : 1));
            first_segment = it + 1 == n_own;      // the shared range starts with a "first" segment again
            if (!last) {
                advance(t_c, uu_c, it + 1);        // a new tile or the jump to the shared range: a new slab either way
                slab_c ^= 1;
                whole = segment_is_whole(t_c, uu_c);
                setup_compute(tile_of(t_c));
            }
        } else {
            ++uu_c;
            if (P.NTR == 1 || uu_c % P.NTR == 0) slab_c ^= 1;
        }
    }
}

}  // namespace mcn
