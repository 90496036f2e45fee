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
#include "kvtc_dev.h"
#include "kvtc_numeric.h"

namespace kvtc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kDecStages = 2;          // basis slabs in the LDS ring

__device__ __forceinline__ bf16x8 as_bf16x8_d(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

template <int NCT, int TT, typename OT>
__device__ __forceinline__ void decode_tile(const PlanDev* __restrict__ P, const TileRef& tr,
                                            const KernelArgs& a, uint4* smem) {
    constexpr int TOK_W = 32 * TT;
    constexpr int TOK_WG = 4 * TOK_W;
    constexpr int SLAB_U4 = 2 * NCT * 64;          // one 32-feature tile of V_kept

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int p = P->p;
    const int T = tr.n_tokens;
    const int tok_tile0 = tr.tile * TOK_WG;
    const int rd = P->rec_dwords;
    const int rstride = rd + 1;

    // ---- records -> LDS (coalesced), then each lane unpacks its blocks ---------------
    uint32_t* rec = reinterpret_cast<uint32_t*>(smem);
    {
        const int n_valid = min(TOK_WG, T - tok_tile0);
        const uint32_t* in = reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(a.stream_buf) + tr.offset) +
                             (size_t)tok_tile0 * rd;
        const uint32_t magic = 0xffffffffu / (uint32_t)rd + 1u;
        const int total = n_valid * rd;
        for (int i = tid; i < total; i += kThreads) {
            const uint32_t t = __umulhi((uint32_t)i, magic);
            rec[t * rstride + ((uint32_t)i - t * rd)] = in[i];
        }
        // pad dwords: defined contents.  Rows past the end of the tensor replicate the last token's
        // record, so every lane decodes something valid and the tail lanes store the same bytes to
        // the same place as the last token's lane: no store is ever predicated off, which keeps the
        // number of memory operations per step fixed (the explicit vmcnt waits count on it).
        for (int i = tid; i < TOK_WG; i += kThreads) rec[i * rstride + rd] = 0u;
        const uint32_t* last = in + (size_t)(n_valid - 1) * rd;
        for (int i = total + tid; i < TOK_WG * rd; i += kThreads) {
            const uint32_t t = __umulhi((uint32_t)i, magic);
            const uint32_t w = (uint32_t)i - t * rd;
            rec[t * rstride + w] = last[w];
        }
    }
    __syncthreads();

    bf16x8 aop[TT][2 * NCT];
#pragma unroll
    for (int c = 0; c < NCT; ++c) {
        const uint32_t info = P->blk[2 * c + h];
        const uint32_t bits = info & 0xffu;
        const uint32_t g = (info >> 8) & 0xffu;
        const uint32_t pos0 = (info >> 16) * 16u;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float d[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) d[i] = 0.0f;
            if (bits != 0u) {
                const uint32_t* row = rec + (wave * TOK_W + tt * 32 + l32) * rstride;
                const uint32_t hdr = row[g];
                const float shift = f16_bits_to_f32((uint16_t)(hdr & 0xffffu));
                const float scale = f16_bits_to_f32((uint16_t)(hdr >> 16));
                if (bits <= 8u) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t pos = pos0 + 4u * k * bits;
                        const uint32_t dw = pos >> 5;
                        const uint32_t w = __builtin_amdgcn_alignbit(row[dw + 1], row[dw], pos & 31u);
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            const uint32_t code = __builtin_amdgcn_ubfe(w, m * bits, bits);
                            d[4 * k + m] = __fmaf_rn((float)code, scale, shift);
                        }
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const uint32_t pos = pos0 + 2u * k * bits;
                        const uint32_t dw = pos >> 5;
                        const uint32_t w = __builtin_amdgcn_alignbit(row[dw + 1], row[dw], pos & 31u);
#pragma unroll
                        for (int m = 0; m < 2; ++m) {
                            const uint32_t code = __builtin_amdgcn_ubfe(w, m * bits, bits);
                            d[2 * k + m] = __fmaf_rn((float)code, scale, shift);
                        }
                    }
                }
            }
            bf16x8 f0, f1;
#pragma unroll
            for (int i = 0; i < 8; ++i) { f0[i] = (__bf16)d[i]; f1[i] = (__bf16)d[8 + i]; }
            aop[tt][2 * c] = f0;
            aop[tt][2 * c + 1] = f1;
        }
    }
    __syncthreads();          // record image is dead; the slabs reuse its space

    // ---- sweep the feature tiles --------------------------------------------------------
    // LDS ring of NSTAGE basis slabs (one 32-feature tile each), filled by asynchronous
    // global->LDS transfers issued NSTAGE-1 tiles ahead.
    constexpr int NSTAGE = kDecStages;
    constexpr int D = NSTAGE - 1;
    constexpr int NV = SLAB_U4 / kThreads;
    static_assert(SLAB_U4 % kThreads == 0, "whole transfers");
    const uint4* vg = uniform_ptr(P->v_dec);
    const int n_ft = p / 32;                                   // even: p is a multiple of 64
    const uint32_t lds_ring = lds_offset(smem);
    auto issue = [&](int ft, int stage) {
        const uint4* vsrc = vg + (size_t)ft * SLAB_U4;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            dma16_async(vsrc + i * kThreads, (uint32_t)tid * 16u,
                        __builtin_amdgcn_readfirstlane(lds_ring + (stage * SLAB_U4 + i * kThreads + wave * 64) * 16));
    };

    // Output addressing.  Accumulator register i of token tile tt holds row tt*32 + 8*(i/4) + 4*h + i%4
    // of this wave's tokens; the lane's two features of a pair of tiles are adjacent in memory.
    // Rows past the end of the tensor are redirected to the last token's row (they hold its values).
    constexpr int NST = 16 * TT;                               // stores per pair of feature tiles, never predicated off
    const uint32_t ldb = (uint32_t)a.ld_x * (uint32_t)sizeof(OT);
    const int n_valid = min(TOK_WG, T - tok_tile0);
    const bool full = n_valid == TOK_WG;
    char* obase = reinterpret_cast<char*>(const_cast<void*>(a.x)) + (size_t)(tr.x_row0 + tok_tile0) * (size_t)a.ld_x * sizeof(OT);
    const uint32_t lane_row = (uint32_t)(wave * TOK_W + 4 * h);
    const uint32_t lane_col = (uint32_t)(2 * l32 * (int)sizeof(OT));
    const uint32_t lane_off = lane_row * ldb + lane_col;
    auto put = [&](char* dst, float even, float odd) {
        if constexpr (sizeof(OT) == 2) *reinterpret_cast<uint32_t*>(dst) = pack_bf16x2(even, odd);
        else *reinterpret_cast<float2*>(dst) = make_float2(even, odd);
    };

    // mu sits in LDS behind the ring: a global load inside the loop would make the compiler
    // wait for everything in flight, the asynchronous transfers included
    float* mu_lds = reinterpret_cast<float*>(smem + NSTAGE * SLAB_U4);
    for (int i = tid; i < p; i += kThreads) mu_lds[i] = P->mu[i];

#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n_ft) issue(u, u);
    wait_vmem_times<NV>(min(D - 1, n_ft - 1));
    __syncthreads();

    for (int f0 = 0; f0 < n_ft; f0 += 2) {
        f32x16 acc[2][TT];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int ft = f0 + e;
            const int stage = NSTAGE == 2 ? e : ft % NSTAGE;
            const bool more = ft + D < n_ft;
            if (more) issue(ft + D, NSTAGE == 2 ? 1 - e : (ft + D) % NSTAGE);
            {
                const float2 m2 = *reinterpret_cast<const float2*>(mu_lds + f0 * 32 + 2 * l32);
                const float m = e ? m2.y : m2.x;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[e][tt][i] = m;
            }
            constexpr int NSTEP = 2 * NCT;
            const uint4* bbase = smem + stage * SLAB_U4 + lane;
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
                    acc[e][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[tt][ks], bv, acc[e][tt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (e == 1) {
                char* ob = obase + (size_t)(f0 / 2) * (64 * sizeof(OT));
                // (lane_off and last_row pass through an empty asm so that the 32 offsets are recomputed
                // here -- one add each -- instead of being hoisted out of the sweep into registers the
                // accumulators need)
                if (full) {
                    uint32_t lo = lane_off;
                    asm volatile("" : "+v"(lo));
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            put(ob + (lo + (uint32_t)(tt * 32 + 8 * (i / 4) + i % 4) * ldb), acc[0][tt][i], acc[1][tt][i]);
                } else {
                    uint32_t last_row = (uint32_t)(n_valid - 1);
                    asm volatile("" : "+v"(last_row));
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const uint32_t row = min(lane_row + (uint32_t)(tt * 32 + 8 * (i / 4) + i % 4), last_row);
                            put(ob + (row * ldb + lane_col), acc[0][tt][i], acc[1][tt][i]);
                        }
                }
            }
            // The slab of the next step must have landed before the barrier publishes it.  Memory
            // operations complete in issue order, so it is enough that no more operations are in
            // flight than were issued after that slab's transfers: the transfers of the D-1 later
            // slabs and the stores of the odd steps among the last D.  Near the end of the sweep
            // fewer transfers are issued, so everything is waited for.
            constexpr int kYoungerEven = (D - 1) * NV + (D / 2) * NST;
            constexpr int kYoungerOdd = (D - 1) * NV + ((D + 1) / 2) * NST;
            if (!more) wait_vmem<0>();
            else if (e == 0) wait_vmem<(kYoungerEven < 63 ? kYoungerEven : 63)>();
            else wait_vmem<(kYoungerOdd < 63 ? kYoungerOdd : 63)>();
            __syncthreads();
        }
    }
}

// Two kernels, as for encode: narrow plans (two token tiles per wave, up to 320 padded
// coordinates) run two workgroups per compute unit, wide ones get the whole register file.
template <typename OT>
__global__ void __launch_bounds__(kThreads, 2) kvtc_decode_kernel(const KernelArgs a) {
    extern __shared__ uint4 smem[];
    uint32_t* tile_start = reinterpret_cast<uint32_t*>(smem);
    uint4* work = smem + kJobTableBytes / 16 + 1;
    const uint32_t total = build_tile_table<false, 0>(a, tile_start, reinterpret_cast<uint32_t*>(work));
    for (uint32_t tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const TileRef tr = find_tile(a, tile_start, tile);
        const PlanDev* P = a.plans + tr.plan;
        const int key = __builtin_amdgcn_readfirstlane(P->dec_tt * 100 + P->dec_nct);
        switch (key) {
#define KVTC_CASE(TT, NCT) case (TT) * 100 + (NCT): decode_tile<NCT, TT, OT>(P, tr, a, work); break;
            KVTC_CASE(2, 2) KVTC_CASE(2, 4) KVTC_CASE(2, 6) KVTC_CASE(2, 8) KVTC_CASE(2, 10)
#undef KVTC_CASE
            default: break;
        }
    }
}

template <typename OT>
__global__ void __launch_bounds__(kThreads, 1) kvtc_decode_wide_kernel(const KernelArgs a) {
    extern __shared__ uint4 smem[];
    uint32_t* tile_start = reinterpret_cast<uint32_t*>(smem);
    uint4* work = smem + kJobTableBytes / 16 + 1;
    const uint32_t total = build_tile_table<false, 1>(a, tile_start, reinterpret_cast<uint32_t*>(work));
    for (uint32_t tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const TileRef tr = find_tile(a, tile_start, tile);
        const PlanDev* P = a.plans + tr.plan;
        const int key = __builtin_amdgcn_readfirstlane(P->dec_tt * 100 + P->dec_nct);
        switch (key) {
#define KVTC_CASE(TT, NCT) case (TT) * 100 + (NCT): decode_tile<NCT, TT, OT>(P, tr, a, work); break;
            KVTC_CASE(1, 12) KVTC_CASE(1, 16) KVTC_CASE(1, 20) KVTC_CASE(1, 24) KVTC_CASE(1, 32)
#undef KVTC_CASE
            default: break;
        }
    }
}

template <typename K>
static hipError_t set_lds_attr_d(K kernel) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
}

hipError_t launch_decode(const KernelArgs& a, kvtc_dtype dtype, int wide, int grid, size_t lds_bytes, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = set_lds_attr_d(&kvtc_decode_kernel<uint16_t>);
        if (e == hipSuccess) e = set_lds_attr_d(&kvtc_decode_kernel<float>);
        if (e == hipSuccess) e = set_lds_attr_d(&kvtc_decode_wide_kernel<uint16_t>);
        if (e == hipSuccess) e = set_lds_attr_d(&kvtc_decode_wide_kernel<float>);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (!wide) {
        if (dtype == KVTC_BF16)
            hipLaunchKernelGGL(kvtc_decode_kernel<uint16_t>, dim3(grid), dim3(kThreads), lds_bytes, stream, a);
        else
            hipLaunchKernelGGL(kvtc_decode_kernel<float>, dim3(grid), dim3(kThreads), lds_bytes, stream, a);
    } else {
        if (dtype == KVTC_BF16)
            hipLaunchKernelGGL(kvtc_decode_wide_kernel<uint16_t>, dim3(grid), dim3(kThreads), lds_bytes, stream, a);
        else
            hipLaunchKernelGGL(kvtc_decode_wide_kernel<float>, dim3(grid), dim3(kThreads), lds_bytes, stream, a);
    }
    return hipGetLastError();
}

int decode_lds_bytes(int nct, int tt, int rec_dwords, int p, kvtc_dtype dtype) {
    const int tok_wg = 4 * 32 * tt;
    const int rec_b = tok_wg * (rec_dwords + 1) * 4;
    const int slab_b = kDecStages * 2 * nct * 1024 + p * 4;
    (void)dtype;
    return rec_b > slab_b ? rec_b : slab_b;
}

}  // namespace kvtc
