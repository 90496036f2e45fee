// Fused decode kernel for gfx950, the mirror of the encode kernel: records are unpacked
// and dequantised straight into bf16 matrix-core operands, back-projected with V_kept and
// un-centred, one launch.  (Paper, Section "Method", mode "Decompression"; eq. 3.)
//
// X_hat = D_hat V_kept^T with the 32x32x16 bf16 MFMA: M = tokens, N = features,
// K = kept coordinates.  In the prologue a lane owns one token: its dequantised coordinates ARE
// its A operand (16 consecutive coordinates = one block of the record = two k-step fragments),
// built once per tile and kept in registers while the wave sweeps the feature tiles.
// V_kept is pre-swizzled into B fragments per 32-feature tile, moved global -> LDS without
// register staging (ring of slabs) and shared by the four wavefronts.  The accumulator then has
// features across lanes and tokens across registers.  Feature tiles come in pairs that
// interleave the even and the odd features of a 64-feature span, so a lane packs its two
// results into one dword (bf16) or one dwordx2 (fp32) and every store instruction writes whole
// 128-byte lines of two token rows -- no transposition through LDS (measured on MI355X: such
// dword stores reach the same 5.7 TB/s as 16-byte stores of whole lines, while pieces of
// 32 bytes per row reach 1.6 TB/s).
#include <hip/hip_runtime.h>
#include <type_traits>
#include "kvtc_dev.h"
#include "kvtc_numeric.h"

namespace kvtc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_bf16x8_d(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Work-area layout in LDS (behind the job table): [block table of the tile's plan, 256 B][record
// image][basis ring].  The ring has two stages; a stage is one 32-feature slab of B fragments
// followed by that tile's 32 entries of mu (kMuU4 * 16 bytes with padding).
constexpr int kDecStages = 2;
constexpr int kMuU4 = 16;
constexpr int kAuxBytes = 256;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Where the records of a tile sit in the LDS image.  Transfers move 16 bytes per lane (the
// global->LDS path handles a lane at a time, so narrower pieces cost the same and carry less):
//   * records of a whole number of 16-byte pieces, the tile starting on a 16-byte boundary of the
//     stream (it does unless jobs with other record sizes precede it): each row gets an odd number of pieces (one or
//     two of padding), which spreads the rows that 32 lanes unpack side by side over the banks
//     (two lanes per bank at worst);
//   * other record sizes: the tile's bytes are copied as they are, starting from the 16-byte
//     boundary below the tile's first byte (`skew` dwords before it); the row stride is then rd
//     dwords, which is not a multiple of four -- again two lanes per bank at worst.
struct RecImage {
    uint32_t stride_dw;     // LDS dwords from one row to the next
    uint32_t skew_dw;       // LDS dwords before row 0
    uint32_t pieces_row;    // padded scheme: pieces per row, padding included; 0 = verbatim copy
};
__device__ __forceinline__ RecImage rec_image(int rd, uint64_t tile_byte0) {
    RecImage im;
    if ((rd & 3) == 0 && (tile_byte0 & 15u) == 0u) {
        const uint32_t m = (uint32_t)rd >> 2;
        im.pieces_row = (m & 1u) ? m + 2u : m + 1u;
        im.stride_dw = 4u * im.pieces_row;
        im.skew_dw = 0u;
    } else {
        im.pieces_row = 0u;
        im.stride_dw = (uint32_t)rd;
        im.skew_dw = (uint32_t)(tile_byte0 & 15u) >> 2;
    }
    return im;
}

// Records of one workgroup tile (and the block table of its plan), global -> LDS, asynchronously
// and without register staging.  Only the tile's valid rows are fetched; rows past the end of the
// tensor are never read (the unpacking redirects them to the last valid row).  Returns the number
// of transfers this wave issued; the caller owns the wait (vmcnt) and the barrier that publishes
// the image.
__device__ __forceinline__ int issue_records(const KernelArgs& a, const TileRef& t, const PlanDec& P, uint32_t lds_work) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rd = P.rec_dwords, tok_wg = P.dec_tok_wg;
    const int tok0 = t.tile * tok_wg;
    const uint32_t n_valid = (uint32_t)min(tok_wg, t.n_tokens - tok0);
    const uint64_t byte0 = t.offset + (uint64_t)tok0 * (uint64_t)rd * 4ull;
    const RecImage im = rec_image(rd, byte0);
    const uint8_t* src = reinterpret_cast<const uint8_t*>(a.stream_buf) + (byte0 & ~15ull);
    const uint32_t lds_rec = lds_work + kAuxBytes;
    int n = 0;
    if (wave == 0) {
        dma4_async(P.blk, (uint32_t)lane * 4u, lds_work);
        ++n;
    }
    if (im.pieces_row != 0u) {
        const uint32_t m = (uint32_t)rd >> 2;
        const uint32_t total = n_valid * im.pieces_row;          // LDS slots, padding included
        const uint32_t magic = 0xffffffffu / im.pieces_row + 1u;
        for (uint32_t l0 = (uint32_t)wave * 64u; l0 < total; l0 += kThreads) {
            const uint32_t l = l0 + (uint32_t)lane;
            if (l < total) {
                const uint32_t row = __umulhi(l, magic);
                const uint32_t col = l - row * im.pieces_row;
                dma16_async(src, (row * m + min(col, m - 1u)) * 16u, lds_rec + l0 * 16u);    // padding repeats the last piece
            }
            ++n;
        }
    } else {
        const uint32_t total = (im.skew_dw * 4u + n_valid * (uint32_t)rd * 4u + 15u) >> 4;   // pieces
        for (uint32_t l0 = (uint32_t)wave * 64u; l0 < total; l0 += kThreads) {
            const uint32_t l = l0 + (uint32_t)lane;
            if (l < total) dma16_async(src, l * 16u, lds_rec + l0 * 16u);
            ++n;
        }
    }
    return n;
}

// One workgroup tile.  The work area holds the tile's block table and record image, landed and
// published.  With `prefetch` the ring does not overlap them: the first basis slab is requested
// before unpacking, and the records of the workgroup's next tile (if any) are requested during
// the first step of the feature sweep.
template <int NCT, int TT, typename OT, int ACC>
__device__ __forceinline__ void decode_tile(const PlanDec& P, const TileRef& tr, const KernelArgs& a, uint4* work, uint4* ring,
                                            bool prefetch, bool has_next, const TileRef& next, const PlanDec& Pn) {
    constexpr int TOK_W = 32 * TT;
    constexpr int TOK_WG = 4 * TOK_W;
    constexpr int SLAB_U4 = 2 * NCT * 64;          // one 32-feature tile of V_kept
    constexpr int STAGE_U4 = SLAB_U4 + kMuU4;
    constexpr int NV = (SLAB_U4 + kThreads - 1) / kThreads;     // transfer rounds of the workgroup per slab; with an odd tile count the last one is half a round (waves 0 and 1)
    static_assert(SLAB_U4 % 128 == 0, "whole wave transfers");
    static_assert(kDecStages == 2, "the wait counts below are written out for a ring of two slabs");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int p = P.p;
    const int T = tr.n_tokens;
    const int tok_tile0 = tr.tile * TOK_WG;
    const int rd = P.rec_dwords;
    const int n_valid = min(TOK_WG, T - tok_tile0);
    const RecImage im = rec_image(rd, tr.offset + (uint64_t)tok_tile0 * (uint64_t)rd * 4ull);
    const int n_ft = p / 32;                                   // even: p is a multiple of 64

    // basis slab of feature tile ft -> ring stage; wave 0 also moves the tile's mu entries
    const uint4* vg = P.v_dec;
    const uint32_t lds_ring = lds_offset(ring);
    auto issue_slab = [&](int ft, int stage) {
        const uint4* vsrc = vg + (size_t)ft * STAGE_U4;
        const uint32_t dst = lds_ring + (uint32_t)(stage * STAGE_U4) * 16u;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (i * kThreads + wave * 64 < SLAB_U4)
                dma16_async(vsrc + i * kThreads, (uint32_t)tid * 16u, dst + (uint32_t)(i * kThreads + wave * 64) * 16u);
        if (wave == 0 && lane < kMuU4) dma16_async(vsrc + SLAB_U4, (uint32_t)lane * 16u, dst + (uint32_t)SLAB_U4 * 16u);
    };
    if (prefetch) issue_slab(0, 0);

    // ---- each lane unpacks its blocks from the record image ------------------------------
    // A lane owns one token (l32) and, per 32-coordinate tile, the 16-coordinate block of its half h.
    const uint32_t* blk = reinterpret_cast<const uint32_t*>(work);
    const uint32_t* rec = blk + kAuxBytes / 4 + im.skew_dw;
    bf16x8 aop[TT][2 * NCT];
    // codes of up to 8 bits (all that calibration produces) come four to a 32-bit window, wider
    // ones two; the choice is made once per plan
    auto unpack = [&](auto narrow_tag) {
        constexpr bool kNarrow = decltype(narrow_tag)::value;
        constexpr int PER = kNarrow ? 4 : 2;                   // codes per window
#pragma unroll
        for (int c = 0; c < NCT; ++c) {
            const uint32_t info = blk[2 * c + h];
            const uint32_t bits = info & 0xffu;
            const uint32_t g = (info >> 8) & 0xffu;
            const uint32_t pos0 = (info >> 16) * 16u;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const uint32_t* row = rec + (uint32_t)min(wave * TOK_W + tt * 32 + l32, n_valid - 1) * im.stride_dw;   // tail rows: the last token's record
                const uint32_t hdr = bits != 0u ? row[g] : 0u;      // a block without bits decodes to zeros
                const float shift = f16_bits_to_f32((uint16_t)(hdr & 0xffffu));
                const float scale = f16_bits_to_f32((uint16_t)(hdr >> 16));
                uint32_t q[8];                                      // the block's 16 values as bf16 pairs
#pragma unroll
                for (int k = 0; k < 16 / PER; ++k) {
                    const uint32_t pos = pos0 + (uint32_t)(PER * k) * bits;
                    const uint32_t dw = pos >> 5;
                    const uint32_t w = __builtin_amdgcn_alignbit(row[dw + 1], row[dw], pos & 31u);
#pragma unroll
                    for (int m = 0; m < PER; m += 2) {
                        const float d0 = __fmaf_rn((float)__builtin_amdgcn_ubfe(w, m * bits, bits), scale, shift);
                        const float d1 = __fmaf_rn((float)__builtin_amdgcn_ubfe(w, (m + 1) * bits, bits), scale, shift);
                        q[(PER * k + m) / 2] = pack_bf16x2(d0, d1);
                    }
                }
                // (through an empty asm: the conversions are done here, block by block, instead of all the
                // fp32 values staying live until the end of the unpacking)
                asm volatile("" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]), "+v"(q[4]), "+v"(q[5]), "+v"(q[6]), "+v"(q[7]));
                aop[tt][2 * c] = __builtin_bit_cast(bf16x8, make_uint4(q[0], q[1], q[2], q[3]));
                aop[tt][2 * c + 1] = __builtin_bit_cast(bf16x8, make_uint4(q[4], q[5], q[6], q[7]));
            }
        }
    };
    if (P.code_bits_max <= 8) unpack(std::true_type()); else unpack(std::false_type());
    if (!prefetch) {
        __syncthreads();          // record image is dead; the ring reuses its space
        issue_slab(0, 0);
    }
    wait_vmem<0>();
    __syncthreads();              // slab 0 is published (and, with prefetch, the record image is dead)

    // ---- sweep the feature tiles --------------------------------------------------------
    // Output addressing.  Accumulator register i of token tile tt holds row tt*32 + 8*(i/4) + 4*h + i%4
    // of this wave's tokens; the lane's two features of a pair of tiles are adjacent in memory.
    // Rows past the end of the tensor are redirected to the last token's row (they hold its values),
    // so no store is ever predicated off and the number of memory operations per step is fixed.
    constexpr int NST = 16 * TT;                               // stores per pair of feature tiles
    const uint32_t ldb = (uint32_t)a.ld_x * (uint32_t)sizeof(OT);
    char* obase = reinterpret_cast<char*>(const_cast<void*>(a.x)) + (size_t)(tr.x_row0 + tok_tile0) * (size_t)a.ld_x * sizeof(OT);
    const uint32_t lane_row = (uint32_t)(wave * TOK_W + 4 * h);
    const uint32_t lane_col = (uint32_t)(2 * l32 * (int)sizeof(OT));
    const uint32_t last_row = (uint32_t)(n_valid - 1);

    // One 32-feature tile: the accumulators start from mu and sweep the coordinates.
    auto tile_step = [&](int stage, f32x16 (&acc)[TT]) {
        const uint4* bbase = ring + stage * STAGE_U4 + lane;
        {
            const float m = reinterpret_cast<const float*>(ring + stage * STAGE_U4 + SLAB_U4)[l32];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tt][i] = m;
        }
        constexpr int NSTEP = 2 * NCT;
        uint4 bf[3];
        bf[0] = bbase[0];
        bf[1] = bbase[64];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < NSTEP; ++ks) {
            if (ks + 2 < NSTEP) bf[(ks + 2) % 3] = bbase[(ks + 2) * 64];
            const bf16x8 bv = as_bf16x8_d(bf[ks % 3]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[tt][ks], bv, acc[tt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Waits: the slab of the next step must have landed before the barrier publishes it.  Memory
    // operations complete in issue order, so it is enough that no more operations are in flight
    // than this wave issued after that slab's transfers (the next tile's records in the first
    // step, the stores in odd steps).
    for (int f0 = 0; f0 < n_ft; f0 += 2) {
        f32x16 acc0[TT], acc1[TT];
        issue_slab(f0 + 1, 1);
        int n_rec = 0;
        if (f0 == 0 && has_next) n_rec = issue_records(a, next, Pn, lds_offset(work));
        tile_step(0, acc0);
        if (f0 == 0) wait_vmem_dyn(n_rec); else wait_vmem<0>();
        __syncthreads();

        const bool more = f0 + 2 < n_ft;
        if (more) issue_slab(f0 + 2, 0);
        tile_step(1, acc1);
        {
            // the 64-feature span f0 / 2 of the token's features; with a blocked layout (heads or layers apart in
            // memory) every whole block before it adds the gap between blocks
            char* ob = obase + (size_t)(f0 / 2) * (64 * sizeof(OT)) +
                       (a.x_blk_log2 ? (size_t)(((f0 / 2) * 64) >> a.x_blk_log2) * ((size_t)a.x_blk_jump * sizeof(OT)) : (size_t)0);
            // (through an empty asm so that the 16*TT offsets are recomputed here -- three vector
            // instructions each -- instead of being hoisted out of the sweep into registers the
            // accumulators need)
            uint32_t lrow = lane_row;
            asm volatile("" : "+v"(lrow));
            if constexpr (ACC == 1) {
                // a further section of a sectioned plan: its part of the product is ADDED to what the earlier
                // sections left in the fp32 output (hardware float adds in memory, nothing returned).  Rows past
                // the tensor's end are skipped, not redirected: adding the last row's values twice would be wrong.
                static_assert(sizeof(OT) == 4, "sections are summed in fp32");
#pragma unroll
                for (int k = 0; k < NST; ++k) {
                    const int tt = k / 16, i = k % 16;
                    const uint32_t row = lrow + (uint32_t)(tt * 32 + 8 * (i / 4) + i % 4);
                    if (row <= last_row) {
                        float* dst = reinterpret_cast<float*>(ob + (__umul24(row, ldb) + lane_col));
                        unsafeAtomicAdd(dst, acc0[tt][i]);
                        unsafeAtomicAdd(dst + 1, acc1[tt][i]);
                    }
                }
            } else if constexpr (ACC == 2) {
                // the last section of a sectioned plan, bf16 output: the earlier sections' fp32 sum (rows of a.dec_sum_ld
                // floats, features contiguous) plus this section's part, rounded to bf16 once and stored at the caller's layout
                static_assert(sizeof(OT) == 2, "the final rounding is to bf16");
                const char* sb = reinterpret_cast<const char*>(a.dec_sum) +
                                 ((size_t)(tr.x_row0 + tok_tile0) * (size_t)a.dec_sum_ld + (size_t)(f0 / 2) * 64) * sizeof(float);
                const uint32_t sld = (uint32_t)a.dec_sum_ld * (uint32_t)sizeof(float);
#pragma unroll
                for (int k = 0; k < NST; ++k) {
                    const int tt = k / 16, i = k % 16;
                    const uint32_t row = lrow + (uint32_t)(tt * 32 + 8 * (i / 4) + i % 4);
                    if (row <= last_row) {
                        const float2 part = *reinterpret_cast<const float2*>(sb + ((size_t)row * sld + 2u * lane_col));
                        *reinterpret_cast<uint32_t*>(ob + (__umul24(row, ldb) + lane_col)) = pack_bf16x2(part.x + acc0[tt][i], part.y + acc1[tt][i]);
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < NST; ++k) {
                    const int tt = k / 16, i = k % 16;
                    const uint32_t row = min(lrow + (uint32_t)(tt * 32 + 8 * (i / 4) + i % 4), last_row);
                    char* dst = ob + (__umul24(row, ldb) + lane_col);              // row < 256, ldb <= 2^23
                    if constexpr (sizeof(OT) == 2) *reinterpret_cast<uint32_t*>(dst) = pack_bf16x2(acc0[tt][i], acc1[tt][i]);
                    else *reinterpret_cast<float2*>(dst) = make_float2(acc0[tt][i], acc1[tt][i]);
                }
            }
        }
        // (the adds are a data-dependent number of operations, so after them the wait is for everything)
        if (more && ACC == 0) wait_vmem<NST>(); else wait_vmem<0>();
        __syncthreads();
    }
}

// One kernel per register class (TT token tiles per wave, plans of up to CLS coordinate tiles): up to 4 tiles
// three workgroups share a compute unit, up to 10 two, up to 18 and up to 24 one with the whole register
// file (two token tiles per wave), beyond that one token tile per wave.  Inside a class every tile runs the
// code of its own plan's width (a switch over the widths built for the class -- their register needs are
// alike, so the class allocates what its widest member needs and no more), which makes a batch whose plans
// differ in width ONE launch per class: separate launches per width each ended with compute units idle
// while their last tiles finished (the 32-layer cache at 16x has plans of 7, 8 and 9 tiles: 1.39 ms in
// three launches, against 16 full rounds of tiles in one).  A batched launch serves only the jobs whose
// plan belongs to its class.  The tile loop is persistent.  With a non-zero a.dec_ring_off the ring sits
// behind the record image and each tile's records are fetched during the previous tile's sweep; with
// offset 0 they share the space and the records are fetched at the tile's start.
// (must agree with the host's class table)
template <int TT, int CLS> constexpr int dec_wgs_per_cu() { return CLS <= 4 ? 3 : (CLS <= 10 ? 2 : 1); }

// The widths built for each class; a plan's tile count is rounded up to the next of them at plan creation.
template <int CLS, int TT, typename OT, int ACC>
__device__ __forceinline__ void decode_tile_of_class(const PlanDec& P, const TileRef& tr, const KernelArgs& a, uint4* work, uint4* ring,
                                                     bool prefetch, bool has_next, const TileRef& next, const PlanDec& Pn) {
#define KVTC_W(N) case N: decode_tile<N, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn); break;
    if constexpr (CLS == 4) {
        switch (P.dec_nct) { KVTC_W(2) default: decode_tile<4, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn); break; }
    } else if constexpr (CLS == 10) {
        switch (P.dec_nct) { KVTC_W(6) KVTC_W(7) KVTC_W(8) KVTC_W(9) default: decode_tile<10, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn); break; }
    } else if constexpr (CLS == 18) {
        switch (P.dec_nct) { KVTC_W(12) KVTC_W(16) KVTC_W(17) default: decode_tile<18, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn); break; }
    } else if constexpr (CLS == 24) {
        switch (P.dec_nct) { KVTC_W(20) default: decode_tile<24, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn); break; }
    } else {
        decode_tile<32, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next, next, Pn);
    }
#undef KVTC_W
}

template <typename OT, int TT, int CLS, int ACC = 0>
__global__ void __launch_bounds__(kThreads, (dec_wgs_per_cu<TT, CLS>())) kvtc_decode_kernel(const KernelArgs a) {
    extern __shared__ uint4 smem[];
    uint32_t* tile_start = reinterpret_cast<uint32_t*>(smem);
    uint4* work = smem + kJobTableBytes / 16 + 1;
    const uint32_t total = build_tile_table<false>(a, TT * 100 + CLS, tile_start, reinterpret_cast<uint32_t*>(work));
    const TileRange mine = my_tiles(total);
    uint32_t tile = mine.first;
    if (tile >= mine.end) return;
    const bool prefetch = a.dec_ring_off != 0u;
    uint4* ring = work + a.dec_ring_off / 16u;
    TileRef tr = find_tile(a, tile_start, tile);
    PlanDec P = load_plan_dec(a.plans + tr.plan);
    P.dec_tok_wg = 4 * 32 * TT;              // this variant's tile (the descriptor holds the bulk variant's)
    issue_records(a, tr, P, lds_offset(work));
    wait_vmem<0>();
    __syncthreads();
    for (;;) {
        const uint32_t next = tile + mine.step;
        const bool has_next = next < mine.end;
        TileRef trn = tr;
        PlanDec Pn = P;
        if (has_next) {
            trn = find_tile(a, tile_start, next);
            Pn = load_plan_dec(a.plans + trn.plan);
            Pn.dec_tok_wg = 4 * 32 * TT;
        }
        decode_tile_of_class<CLS, TT, OT, ACC>(P, tr, a, work, ring, prefetch, has_next && prefetch, trn, Pn);
        if (!has_next) break;
        tile = next;
        tr = trn;
        P = Pn;
        if (!prefetch) {
            issue_records(a, tr, P, lds_offset(work));
            wait_vmem<0>();
            __syncthreads();
        }
    }
}

// (token tiles per wave, class): the bulk kernels, then the same classes with one token tile per wave (128-token
// workgroup tiles) for single tensors short enough to run all their tiles at once -- a workgroup without a
// neighbour is bound by its own instruction stream, and this halves it
#define KVTC_DEC_VARIANTS(X) X(2, 4) X(2, 10) X(2, 18) X(2, 24) X(1, 32) X(1, 4) X(1, 10) X(1, 18) X(1, 24)

// key = 100 * TT + CLS
hipError_t launch_decode(const KernelArgs& a, kvtc_dtype dtype, int key, int grid, size_t lds_bytes, hipStream_t stream) {
    const void* fn = nullptr;
    switch (key) {
#define KVTC_X(TT, CLS)                                                                                        \
    case (TT) * 100 + (CLS):                                                                                   \
        if (dtype == KVTC_BF16)                                                                                \
            fn = a.dec_accumulate == 2 ? reinterpret_cast<const void*>(&kvtc_decode_kernel<uint16_t, TT, CLS, 2>) \
                                       : reinterpret_cast<const void*>(&kvtc_decode_kernel<uint16_t, TT, CLS>); \
        else                                                                                                   \
            fn = a.dec_accumulate == 1 ? reinterpret_cast<const void*>(&kvtc_decode_kernel<float, TT, CLS, 1>) \
                                       : reinterpret_cast<const void*>(&kvtc_decode_kernel<float, TT, CLS>);   \
        break;
        KVTC_DEC_VARIANTS(KVTC_X)
#undef KVTC_X
        default: return hipErrorInvalidValue;
    }
    hipError_t e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    KernelArgs args = a;
    void* params[] = {&args};
    return hipLaunchKernel(fn, dim3(grid), dim3(kThreads), params, lds_bytes, stream);
}

// Bytes of the block table + record image and of the basis ring of a decode variant (the host
// lays them out: side by side when both fit, else sharing the space).
int decode_rec_bytes(int tt, int rec_dwords) {
    const int tok_wg = 4 * 32 * tt;
    return kAuxBytes + (tok_wg * (rec_dwords + 8) * 4 + 16 + 1023) / 1024 * 1024;      // padded rows or skew + one piece; whole 64-piece transfers
}
int decode_ring_bytes(int nct) { return kDecStages * (2 * nct * 64 + kMuU4) * 16; }
int decode_stage_u4(int nct) { return 2 * nct * 64 + kMuU4; }

}  // namespace kvtc
