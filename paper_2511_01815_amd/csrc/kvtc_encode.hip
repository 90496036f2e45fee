// Fused encode kernel for gfx950: projection onto the kept PCA basis on the bf16 matrix
// cores, then per-token group min-max quantisation and bit-packing, one launch.
// (Paper, Section "Method", mode "Compression"; Sections "Feature decorrelation" and
// "Quantization".)
//
// Work decomposition.  A workgroup (4 wavefronts, or 8 for plans of 321..640 padded coordinates)
// owns a tile of tokens and ALL kept coordinates of those tokens, because a group's min/max
// needs every coordinate of the group before any of its codes exists.
// The product is computed transposed, D^T = V_kept^T X^T, with the 32x32x16 bf16 MFMA:
// M = coordinates, N = tokens, K = features.  Then a lane owns one token (column) and, by
// permuting the rows of the A operand, 16 *consecutive* coordinates of it per 32-coordinate
// tile -- exactly one 16-coordinate block of the record format, so quantisation and packing
// are lane-local with static bit offsets.
//   * V_kept is pre-swizzled at plan creation into A-operand fragments.  Slabs of it and the
//     matching columns of the tile's X rows move global -> LDS without register staging, a ring
//     stage or two ahead of the MFMAs; every byte of X is read from HBM once, the basis slabs
//     are re-read (from L2) once per tile, so larger token tiles mean less traffic per token.
//   * The coordinates are split over WC wavefronts that share the tokens; the other wavefronts
//     take further tokens.  A wavefront holds TT x NTW accumulator tiles of 32 x 32.
// Epilogue: block min/max -> LDS -> per (token, group) header (fp16 shift down, scale up)
// -> codes -> written into the record image in LDS -> one contiguous, coalesced store of the
// tile's records.
#include <hip/hip_runtime.h>
#include "kvtc_dev.h"
#include "kvtc_numeric.h"

namespace kvtc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// The X slab of one step in LDS: TOK rows of KS*16 features, written by global->LDS transfers
// in 16-byte columns.  Column c of row r is stored at column c ^ swz(r) so that the 8 lanes
// served together by a 128-bit LDS read (8 consecutive tokens, same column) fall on 8 different
// 16-byte bank groups.
template <typename XT, int KS> struct XSlab;
template <int KS> struct XSlab<uint16_t, KS> {                 // bf16 input: KS*32 bytes per row
    static constexpr int ROW_B = KS * 32, COLS = ROW_B / 16, ROWS_PER_DMA = 64 / COLS;
    static __device__ __forceinline__ int swz(int r) { return (r * COLS / 8) & (COLS - 1); }
    // B fragment of (row, k-step, lane half): 8 consecutive features
    static __device__ __forceinline__ bf16x8 frag(const char* slab, int row, int ks, int h) {
        const int c = (2 * ks + h) ^ swz(row);
        return as_bf16x8(*reinterpret_cast<const uint4*>(slab + row * ROW_B + c * 16));
    }
};
template <int KS> struct XSlab<float, KS> {                    // fp32 input: KS*64 bytes per row
    static constexpr int ROW_B = KS * 64, COLS = ROW_B / 16, ROWS_PER_DMA = 64 / COLS;
    static __device__ __forceinline__ int swz(int r) { return (r * COLS / 8) & (COLS - 1); }
    static __device__ __forceinline__ bf16x8 frag(const char* slab, int row, int ks, int h) {
        const int c0 = (4 * ks + 2 * h) ^ swz(row), c1 = (4 * ks + 2 * h + 1) ^ swz(row);
        const float4 a = *reinterpret_cast<const float4*>(slab + row * ROW_B + c0 * 16);
        const float4 b = *reinterpret_cast<const float4*>(slab + row * ROW_B + c1 * 16);
        bf16x8 r;                                                // round to bf16, nearest even
        r[0] = (__bf16)a.x; r[1] = (__bf16)a.y; r[2] = (__bf16)a.z; r[3] = (__bf16)a.w;
        r[4] = (__bf16)b.x; r[5] = (__bf16)b.y; r[6] = (__bf16)b.z; r[7] = (__bf16)b.w;
        return r;
    }
};

// OR `len` bits of v into the record image at bit position pos (pos, len per lane).
__device__ __forceinline__ void put_bits(uint32_t* rec, uint32_t pos, uint32_t v, uint32_t len) {
    const uint32_t dw = pos >> 5, s = pos & 31u;
    atomicOr(rec + dw, v << s);
    if (s + len > 32u) atomicOr(rec + dw + 1, v >> (32u - s));
}

// The 16 codes of a block, BITS wide each, as a bit string of BITS halfwords written to the record
// image at a halfword address (blocks start and end on halfword boundaries: 16 codes x BITS bits).
// Plain 16-bit LDS stores: two blocks may share a dword but never a halfword, so nothing is OR-ed
// and the image needs no clearing.
template <int BITS>
__device__ __forceinline__ void emit_block(const uint32_t (&c)[16], char* dst) {
    uint32_t q[(BITS + 1) / 2];
#pragma unroll
    for (int j = 0; j < (BITS + 1) / 2; ++j) q[j] = 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int pos = i * BITS, dw = pos >> 5, sh = pos & 31;
        q[dw] |= c[i] << sh;
        if (sh + BITS > 32) q[dw + 1] |= c[i] >> (32 - sh);
    }
#pragma unroll
    for (int j = 0; j < BITS; ++j)
        *reinterpret_cast<uint16_t*>(dst + 2 * j) = (uint16_t)(q[j >> 1] >> (16 * (j & 1)));
}

// k-steps (16 features each) per pipeline stage, and stages in the LDS ring.  Sized so that a
// narrow plan (<= 10 coordinate tiles, two workgroups per compute unit) stays within ~72 KB
// and a wide one (one workgroup) within ~150 KB.
// token tiles (of 32) per wave: three where the registers allow it (8 coordinate tiles over two
// waves: 192 accumulator registers), which cuts the basis traffic per token by a third
__host__ __device__ constexpr int enc_tt(int ntp, int nw, int wc) { return nw == 4 && wc == 2 && ntp == 8 ? 3 : 2; }
__host__ __device__ constexpr int enc_ks(int ntp, int elem_bytes) {
    return ntp < 8 || (ntp == 8 && elem_bytes == 2) || (ntp > 10 && ntp <= (elem_bytes == 2 ? 20 : 16)) ? 2 : 1;      // fp32 X slabs are twice as large
}
// stages: as many as fit the variant's LDS share (three workgroups per compute unit: ~44 KB, two: ~72 KB, one: ~150 KB), 2..4
__host__ __device__ constexpr int enc_stages(int ntp, int elem_bytes, int nw, int wc) {
    const int ks = enc_ks(ntp, elem_bytes);
    const int stage_b = ks * ntp * 1024 + 32 * enc_tt(ntp, nw, wc) * (nw / wc) * ks * 16 * elem_bytes;
    const int budget = (nw == 4 && wc == 2 && ntp == 6 ? 44 : (nw == 4 && ntp <= 10 ? 72 : 150)) * 1024;
    const int n = budget / stage_b;
    return n < 2 ? 2 : (n > 4 ? 4 : n);
}

// LDS work area (behind the job table): [tables of the tile's plan: block table 64 dwords, group
// table 64 dwords, -(mu^T V_kept) of the padded coordinates][ring / epilogue images].  The tables
// arrive by asynchronous transfers at the start of a tile, ahead of the first ring stage, so
// no load of the tile loop is visible to the compiler (a visible vector load makes it wait for
// everything in flight, and costs an L2 round trip where it stands).
constexpr int kEncBlkOff = 0, kEncGrpOff = 256, kEncNegcOff = 512;
__host__ __device__ constexpr int enc_aux_bytes(int ntp) { return 512 + ntp * 32 * 4; }

template <int NTW, int WC, typename XT, int NW>
__device__ __forceinline__ void encode_tile(const PlanEnc& P, const TileRef& tr,
                                            const KernelArgs& a, uint4* work) {
    constexpr int NTP = NTW * WC;            // coordinate tiles of the padded plan
    constexpr int TT = enc_tt(NTP, NW, WC);  // token tiles (of 32) per wave
    constexpr int NTH = NW * 64;             // threads of the workgroup
    constexpr int WT = NW / WC;              // waves across tokens
    constexpr int TOK_WG = 32 * TT * WT;
    constexpr int KS = enc_ks(NTP, (int)sizeof(XT));
    constexpr int NSTAGE = enc_stages(NTP, (int)sizeof(XT), NW, WC);
    constexpr int SLAB_U4 = KS * NTP * 64;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = wave % WC, wt = wave / WC;
    const int l32 = lane & 31, h = lane >> 5;
    const int p = P.p;
    const int T = tr.n_tokens;
    const int tok_tile0 = tr.tile * TOK_WG;
    uint4* smem = work + enc_aux_bytes(NTP) / 16;

    // ---- the plan's tables -> LDS (first used in the epilogue) --------------------------
    {
        const uint32_t aux = lds_offset(work);
        if (wave == 0) dma4_async(P.blk, (uint32_t)lane * 4u, aux + kEncBlkOff);
        if (wave == 1) dma4_async(P.grp, (uint32_t)lane * 4u, aux + kEncGrpOff);       // 64 entries allocated
        static_assert(NTP * 8 <= NTH, "one 16-byte piece per thread covers -(mu^T V_kept)");
        if (wave * 64 < NTP * 8 && tid < NTP * 8)
            dma16_async(P.negc, (uint32_t)tid * 16u, aux + kEncNegcOff + (uint32_t)wave * 1024u);
    }

    f32x16 acc[TT][NTW];

    // ---- LDS: a ring of NSTAGE stages, each one basis slab and one X slab ----------
    using XS = XSlab<XT, KS>;
    constexpr int XSLAB_B = TOK_WG * XS::ROW_B;
    constexpr int STAGE_B = SLAB_U4 * 16 + XSLAB_B;
    constexpr int NX_TOTAL = TOK_WG / XS::ROWS_PER_DMA;         // X transfers per stage, dealt round-robin to the waves
    constexpr int NXD = (NX_TOTAL + NW - 1) / NW;
    constexpr int NV_TOTAL = SLAB_U4 / 64;                      // basis transfers per stage (1 KB each), dealt the same way
    constexpr int NV = (NV_TOTAL + NW - 1) / NW;
    constexpr int NDMA_MIN = NV_TOTAL / NW + NX_TOTAL / NW;     // transfers per wave per stage, lower bound over waves
    static_assert(TOK_WG % XS::ROWS_PER_DMA == 0, "whole transfers");
    static_assert(3 * (NV + NXD) < 64, "vmcnt range");
    static_assert(NW >= 2, "waves 0 and 1 fetch the plan's tables");
    char* ring = reinterpret_cast<char*>(smem);
    const uint4* vg = P.v_enc;
    const int n_slabs = p / (16 * KS);

    // per-lane source of each X transfer: row (clamped at the tensor's end) and swizzled column
    const char* xsrc[NXD];
    uint32_t xdst[NXD];                                         // wave-uniform LDS byte offsets inside an X slab
#pragma unroll
    for (int j = 0; j < NXD; ++j) {
        const int row0 = (j * NW + wave) * XS::ROWS_PER_DMA;
        const int row = row0 + lane / XS::COLS;
        const int col = (lane % XS::COLS) ^ XS::swz(row);
        int t = tok_tile0 + row;
        t = t < T ? t : T - 1;                                  // tail rows re-read the last token
        xsrc[j] = reinterpret_cast<const char*>(reinterpret_cast<const XT*>(a.x) + (tr.x_row0 + t) * a.ld_x) + col * 16;
        xdst[j] = (uint32_t)(SLAB_U4 * 16 + row0 * XS::ROW_B);
    }
    const uint32_t lds_ring = lds_offset(ring);

    // All global traffic of the main loop is asynchronous global->LDS transfers issued
    // NSTAGE-1 steps ahead; the only wait is the one in front of the barrier that publishes
    // the next stage, and it leaves the younger stages in flight.
    // byte offset of slab s inside a token's features: KS * 16 features per slab; with a blocked layout
    // (heads or layers apart in memory) every whole block before it adds the gap between blocks
    const int blk_lg = a.x_blk_log2;
    const size_t blk_jump_b = (size_t)a.x_blk_jump * sizeof(XT);
    auto issue = [&](int s, int stage) {
        const uint32_t base = lds_ring + stage * STAGE_B;
        const size_t xoff = (size_t)s * XS::ROW_B + (blk_lg ? (size_t)((s * (16 * KS)) >> blk_lg) * blk_jump_b : (size_t)0);
        const uint4* vsrc = vg + (size_t)s * SLAB_U4 + wave * 64 + lane;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (i * NW + wave < NV_TOTAL)
                dma16_async(vsrc + i * NTH, __builtin_amdgcn_readfirstlane(base + (i * NTH + wave * 64) * 16));
#pragma unroll
        for (int j = 0; j < NXD; ++j)
            if (j * NW + wave < NX_TOTAL)
                dma16_async(xsrc[j] + xoff, __builtin_amdgcn_readfirstlane(base + xdst[j]));
    };
    auto compute = [&](int stage) {
        const uint4* abase = reinterpret_cast<const uint4*>(ring + stage * STAGE_B) + (wc * NTW) * 64 + lane;
        const char* xs = ring + stage * STAGE_B + SLAB_U4 * 16;
        constexpr int NSTEP = KS * NTW;
        bf16x8 xv[KS][TT];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) xv[ks][tt] = XS::frag(xs, (wt * TT + tt) * 32 + l32, ks, h);
        uint4 af[3];
        af[0] = abase[0];
        if (NSTEP > 1) af[1] = abase[((1 / NTW) * NTP + (1 % NTW)) * 64];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NSTEP; ++j) {
            const int ks = j / NTW, ct = j % NTW;
            if (j + 2 < NSTEP) af[(j + 2) % 3] = abase[(((j + 2) / NTW) * NTP + ((j + 2) % NTW)) * 64];
            const bf16x8 av = as_bf16x8(af[j % 3]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[tt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, xv[ks][tt], acc[tt][ct], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    constexpr int D = NSTAGE - 1;                               // prefetch distance in steps
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n_slabs) issue(u, u);
    wait_vmem_times<NDMA_MIN>(min(D - 1, n_slabs - 1));         // stage 0 has landed, and the tables before it
    __syncthreads();

    // ---- accumulators start at -(mu^T V_kept): centring folded into the product ------
    {
        const float* negc = reinterpret_cast<const float*>(work) + kEncNegcOff / 4 + (wc * NTW) * 32 + 16 * h;
#pragma unroll
        for (int ct = 0; ct < NTW; ++ct) {
            f32x16 c;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = *reinterpret_cast<const float4*>(negc + ct * 32 + 4 * q);
                c[4 * q] = v.x; c[4 * q + 1] = v.y; c[4 * q + 2] = v.z; c[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[tt][ct] = c;
        }
    }
    for (int s0 = 0; s0 < n_slabs; s0 += NSTAGE) {
#pragma unroll
        for (int u = 0; u < NSTAGE; ++u) {
            const int s = s0 + u;
            if (s < n_slabs) {
                // stage (u + D) % NSTAGE was read in step s - 1; the barrier that ended it frees it
                if (s + D < n_slabs) issue(s + D, (u + D) % NSTAGE);
                compute(u);
                wait_vmem_times<NDMA_MIN>(min(D - 1, n_slabs - 2 - s));   // stage of step s + 1 has landed
                __syncthreads();
            }
        }
    }

    // ---- epilogue -----------------------------------------------------------------
    // LDS: mm[2*NTP][TOK_WG] float2 | gq[G][TOK_WG] float2 | rec[TOK_WG][rd + 1] dwords
    const int G = P.n_groups;
    const int rd = P.rec_dwords;
    const uint32_t* blk_t = reinterpret_cast<const uint32_t*>(work) + kEncBlkOff / 4;
    const uint32_t* grp_t = reinterpret_cast<const uint32_t*>(work) + kEncGrpOff / 4;
    const int rstride = rd + 1;                 // odd-ish pitch keeps lanes on distinct banks
    float2* mm = reinterpret_cast<float2*>(smem);
    float2* gq = mm + 2 * NTP * TOK_WG;
    uint32_t* rec = reinterpret_cast<uint32_t*>(gq + G * TOK_WG);

    // A: block min/max
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int tw = (wt * TT + tt) * 32 + l32;
#pragma unroll
        for (int ct = 0; ct < NTW; ++ct) {
            const f32x16& d = acc[tt][ct];
            float lo = d[0], hi = d[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) { lo = fminf(lo, d[i]); hi = fmaxf(hi, d[i]); }
            mm[(2 * (wc * NTW + ct) + h) * TOK_WG + tw] = make_float2(lo, hi);
            __builtin_amdgcn_sched_barrier(0);      // keep the accumulator reads from piling up
        }
    }
    // codes wider than 8 bits are OR-ed into the image (cleared here); the usual widths are stored
    const bool narrow_codes = P.code_bits_max <= 8;
    if (!narrow_codes)
        for (int i = tid; i < TOK_WG * rstride; i += NTH) rec[i] = 0u;
    __syncthreads();

    // B: one header per (token, group)
    for (int item = tid; item < TOK_WG * G; item += NTH) {
        const int tw = item % TOK_WG, g = item / TOK_WG;
        const uint32_t gi = grp_t[g];
        const int b0 = gi & 0xff, nb = (gi >> 8) & 0xff, bits = (gi >> 16) & 0xff;
        float lo = __builtin_inff(), hi = -__builtin_inff();
        for (int k = 0; k < nb; ++k) {
            const float2 m = mm[(b0 + k) * TOK_WG + tw];
            lo = fminf(lo, m.x);
            hi = fmaxf(hi, m.y);
        }
        const GroupQ q = group_header(lo, hi, bits);
        gq[g * TOK_WG + tw] = make_float2(q.shift, q.inv);
        rec[tw * rstride + g] = (uint32_t)q.shift16 | ((uint32_t)q.scale16 << 16);
        if (g == 0 && narrow_codes) rec[tw * rstride + rd - 1] = 0u;      // the padding behind the last block
    }
    __syncthreads();

    // C: codes of the lane's blocks, OR-ed into the record image
#pragma unroll
    for (int ct = 0; ct < NTW; ++ct) {
        const uint32_t info = blk_t[2 * (wc * NTW + ct) + h];
        const uint32_t bits = info & 0xffu;
        if (bits != 0u) {
            const uint32_t g = (info >> 8) & 0xffu;
            const uint32_t pos0 = (info >> 16) * 16u;
            const float qmax = (float)((1u << bits) - 1u);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const int tw = (wt * TT + tt) * 32 + l32;
                const float2 sq = gq[g * TOK_WG + tw];
                uint32_t* row = rec + tw * rstride;
                const f32x16& d = acc[tt][ct];
                uint32_t c[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) c[i] = (uint32_t)code_of(d[i], sq.x, sq.y, qmax);
                if (narrow_codes) {
                    char* dst = reinterpret_cast<char*>(row) + (pos0 >> 3);
                    switch (bits) {
                        case 1: emit_block<1>(c, dst); break;
                        case 2: emit_block<2>(c, dst); break;
                        case 3: emit_block<3>(c, dst); break;
                        case 4: emit_block<4>(c, dst); break;
                        case 5: emit_block<5>(c, dst); break;
                        case 6: emit_block<6>(c, dst); break;
                        case 7: emit_block<7>(c, dst); break;
                        default: emit_block<8>(c, dst); break;
                    }
                } else if (bits <= 8u) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t v = c[4 * k] | (c[4 * k + 1] << bits) | (c[4 * k + 2] << (2u * bits)) |
                                           (c[4 * k + 3] << (3u * bits));
                        put_bits(row, pos0 + 4u * k * bits, v, 4u * bits);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const uint32_t v = c[2 * k] | (c[2 * k + 1] << bits);
                        put_bits(row, pos0 + 2u * k * bits, v, 2u * bits);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();

    // D: the tile's records are contiguous in the stream: one coalesced copy, 16 bytes per lane when the
    // tile starts on a 16-byte boundary of the buffer and records are whole 16-byte pieces (then a piece
    // never straddles two rows of the image), else dword by dword
    {
        const int n_valid = min(TOK_WG, T - tok_tile0);
        uint32_t* out = reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(a.stream_buf) + tr.offset) +
                        (size_t)tok_tile0 * rd;
        const uint32_t magic = 0xffffffffu / (uint32_t)rd + 1u;     // exact floor(i / rd) for i < 2^20
        const int total = n_valid * rd;
        if ((rd & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0u) {
            for (int i = 4 * tid; i < total; i += 4 * NTH) {
                const uint32_t t = __umulhi((uint32_t)i, magic);
                const uint32_t* src = rec + t * rstride + ((uint32_t)i - t * rd);
                *reinterpret_cast<uint4*>(out + i) = make_uint4(src[0], src[1], src[2], src[3]);
            }
        } else {
            for (int i = tid; i < total; i += NTH) {
                const uint32_t t = __umulhi((uint32_t)i, magic);
                out[i] = rec[t * rstride + ((uint32_t)i - t * rd)];
            }
        }
    }
    __syncthreads();
}

// One kernel per variant (WC waves across coordinates, NTW coordinate tiles per wave, NW waves per
// workgroup): plans of up to 320 padded coordinates fit 4-wave workgroups with 256 registers per lane,
// two per compute unit (one hides the other's memory waits and epilogue); wider plans get the compute
// unit to themselves, as 8 waves of 256 registers or 4 of 512.  A batched launch serves only the jobs
// whose plan uses its variant.
// (must agree with the host's variant table)
template <int WC, int NTW, int NW> constexpr int enc_wgs_per_cu() {
    return NW == 4 && WC == 2 && NTW == 3 ? 3 : (NW == 4 && WC * NTW <= 10 ? 2 : 1);
}

template <typename XT, int WC, int NTW, int NW>
__global__ void __launch_bounds__(NW * 64, (enc_wgs_per_cu<WC, NTW, NW>())) kvtc_encode_kernel(const KernelArgs a) {
    extern __shared__ uint4 smem[];
    uint32_t* tile_start = reinterpret_cast<uint32_t*>(smem);
    uint4* work = smem + kJobTableBytes / 16 + 1;
    const uint32_t total = build_tile_table<true, NW * 64>(a, NW * 10000 + WC * 100 + NTW, tile_start, reinterpret_cast<uint32_t*>(work));
    const TileRange mine = my_tiles(total);
    for (uint32_t tile = mine.first; tile < mine.end; tile += mine.step) {
        const TileRef tr = find_tile(a, tile_start, tile);
        const PlanEnc P = load_plan_enc(a.plans + tr.plan);
        encode_tile<NTW, WC, XT, NW>(P, tr, a, work);
    }
}

// (waves across coordinates, coordinate tiles per wave, waves per workgroup): the bulk variants, then
// the variants for short jobs -- one wave across the tokens, so a 64-token tile and a third of the
// MFMAs per ring step of the widest bulk tile; a workgroup that has a compute unit to itself (a
// launch of a few short jobs) is bound by exactly those.  The two widest plans' bulk variants
// already have 64-token tiles.
#define KVTC_ENC_VARIANTS(X)                                                                           \
    X(1, 2, 4) X(1, 4, 4) X(2, 3, 4) X(2, 4, 4) X(2, 5, 4) X(4, 3, 8) X(4, 4, 8) X(4, 5, 8) X(4, 6, 4) X(4, 8, 4) \
    X(2, 1, 2) X(4, 1, 4) X(2, 3, 2) X(4, 2, 4) X(2, 5, 2) X(4, 3, 4) X(4, 4, 4) X(4, 5, 4)

// key = 10000 * NW + 100 * WC + NTW
hipError_t launch_encode(const KernelArgs& a, kvtc_dtype dtype, int key, int grid, size_t lds_bytes, hipStream_t stream) {
    const void* fn = nullptr;
    int threads = 0;
    switch (key) {
#define KVTC_X(WC, NTW, NW)                                                                                    \
    case (NW) * 10000 + (WC) * 100 + (NTW):                                                                    \
        fn = dtype == KVTC_BF16 ? reinterpret_cast<const void*>(&kvtc_encode_kernel<uint16_t, WC, NTW, NW>)    \
                                : reinterpret_cast<const void*>(&kvtc_encode_kernel<float, WC, NTW, NW>);      \
        threads = (NW) * 64;                                                                                   \
        break;
        KVTC_ENC_VARIANTS(KVTC_X)
#undef KVTC_X
        default: return hipErrorInvalidValue;
    }
    hipError_t e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    KernelArgs args = a;
    void* params[] = {&args};
    return hipLaunchKernel(fn, dim3(grid), dim3(threads), params, lds_bytes, stream);
}

int encode_tok_wg(int ntw, int wc, int nw) { return 32 * enc_tt(ntw * wc, nw, wc) * (nw / wc); }

// LDS bytes encode_tile needs for a variant (main loop slabs vs epilogue images).
int encode_lds_bytes(int ntw, int wc, int nw, int n_groups, int rec_dwords, kvtc_dtype dtype) {
    const int ntp = ntw * wc;
    const int eb = dtype == KVTC_BF16 ? 2 : 4;
    const int ks = enc_ks(ntp, eb);
    const int tok_wg = 32 * enc_tt(ntp, nw, wc) * (nw / wc);
    const int main_b = enc_stages(ntp, eb, nw, wc) * (ks * ntp * 1024 + tok_wg * ks * (dtype == KVTC_BF16 ? 32 : 64));
    const int epi_b = tok_wg * (2 * ntp * 8 + n_groups * 8 + (rec_dwords + 1) * 4);
    return enc_aux_bytes(ntp) + (main_b > epi_b ? main_b : epi_b);
}

}  // namespace kvtc
