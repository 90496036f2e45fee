// Fused decode kernel for gfx950, the mirror of the encode kernel: records are unpacked
// and dequantised straight into bf16 matrix-core operands, back-projected with V_kept and
// un-centred, one launch.  (Paper, Section "Method", mode "Decompression"; eq. 3.)
//
// X_hat^T = V_kept D_hat^T with the 32x32x16 bf16 MFMA: M = features, N = tokens,
// K = kept coordinates.  A lane owns one token; its dequantised coordinates ARE its B operand
// (16 consecutive coordinates = one block of the record = two k-step fragments), so they are
// built once per tile and stay in registers while the wave sweeps the feature tiles.
// V_kept is pre-swizzled into A fragments per 32-feature tile, moved global -> LDS without
// register staging (double-buffered) and shared by the four wavefronts.  Rows of the A operand are permuted
// so that a lane ends up with 16 consecutive features of its token: 32 contiguous bytes of
// bf16 output per store pair.
#include <hip/hip_runtime.h>
#include "kvtc_dev.h"
#include "kvtc_numeric.h"

namespace kvtc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ bf16x8 as_bf16x8_d(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Output staging.  A lane holds 16 consecutive features of ONE token per (token tile, feature
// tile); storing that directly scatters 16-byte pieces over 32 rows per instruction, and stores
// narrower than a 128-byte line run at a fraction of the write bandwidth (measured on MI355X:
// 16 B pieces 1.3 TB/s, 64 B 3.5 TB/s, whole lines 5.6 TB/s).  Each wave therefore transposes
// through a private LDS tile [tokens][128 bytes] -- one feature tile of fp32 output, two of bf16
// output: lanes write their pieces (16-byte columns, XOR-swizzled against bank conflicts), then
// read back so that 8 consecutive lanes cover one row's 128 bytes, and store whole lines.
template <typename OT> struct OutStage {
    static constexpr int ROW_B = 128;
    static constexpr int FT_PER_ROW = ROW_B / (32 * (int)sizeof(OT));   // feature tiles per line: 2 (bf16), 1 (fp32)
    static constexpr int COLS = ROW_B / 16;                    // 16-byte columns per row
    static constexpr int RPI = 64 / COLS;                      // rows per store instruction
    static __device__ __forceinline__ int swz(int r) { return r & 7; }
};
// `half` = feature tile parity (which 32 of the 64 features)
__device__ __forceinline__ void stage_put(char* st, int row, int h, int half, const f32x16& v, uint16_t) {
    using S = OutStage<uint16_t>;
    uint4 a, b;
    a.x = pack_bf16x2(v[0], v[1]);   a.y = pack_bf16x2(v[2], v[3]);
    a.z = pack_bf16x2(v[4], v[5]);   a.w = pack_bf16x2(v[6], v[7]);
    b.x = pack_bf16x2(v[8], v[9]);   b.y = pack_bf16x2(v[10], v[11]);
    b.z = pack_bf16x2(v[12], v[13]); b.w = pack_bf16x2(v[14], v[15]);
    char* r = st + row * S::ROW_B;
    const int c = 4 * half + 2 * h;
    *reinterpret_cast<uint4*>(r + ((c ^ S::swz(row)) * 16)) = a;
    *reinterpret_cast<uint4*>(r + (((c + 1) ^ S::swz(row)) * 16)) = b;
}
__device__ __forceinline__ void stage_put(char* st, int row, int h, int half, const f32x16& v, float) {
    using S = OutStage<float>;
    char* r = st + row * S::ROW_B;
    const int c = 4 * h;        // one feature tile fills the line
    (void)half;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(r + (((c + q) ^ S::swz(row)) * 16)) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}

template <int NCT, int TT, typename OT>
__device__ __forceinline__ void decode_tile(const PlanDev* __restrict__ P, const TileRef& tr,
                                            const KernelArgs& a, uint4* smem) {
    constexpr int TOK_W = 32 * TT;
    constexpr int TOK_WG = 4 * TOK_W;
    constexpr int SLAB_U4 = 2 * NCT * 64;          // one 32-feature tile of V_kept

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    bf16x8 bop[TT][2 * NCT];
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
            bop[tt][2 * c] = f0;
            bop[tt][2 * c + 1] = f1;
        }
    }
    __syncthreads();          // record image is dead; the slabs reuse its space

    // ---- sweep the feature tiles --------------------------------------------------------
    // LDS ring of NSTAGE basis slabs (one 32-feature tile each), filled by asynchronous
    // global->LDS transfers issued NSTAGE-1 tiles ahead.
    constexpr int NSTAGE = 2;
    constexpr int D = NSTAGE - 1;
    constexpr int NV = SLAB_U4 / kThreads;
    static_assert(SLAB_U4 % kThreads == 0, "whole transfers");
    const uint4* vg = P->v_dec;
    const int n_ft = p / 32;
    const uint32_t lds_ring = lds_offset(smem);
    auto issue = [&](int ft, int stage) {
        const uint4* vsrc = vg + (size_t)ft * SLAB_U4 + wave * 64 + lane;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            dma16_async(vsrc + i * kThreads,
                        __builtin_amdgcn_readfirstlane(lds_ring + (stage * SLAB_U4 + i * kThreads + wave * 64) * 16));
    };

    using OS = OutStage<OT>;
    // store instruction k of a step covers rows k*RPI .. of this wave's 64 tokens; lane -> (row, column)
    constexpr int NS = TOK_W / OS::RPI;                        // store instructions per PAIR of steps (never predicated off)
    char* orow[NS];
    int srow[NS];
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        srow[k] = k * OS::RPI + lane / OS::COLS;
        int t = tok_tile0 + wave * TOK_W + srow[k];
        t = t < T ? t : T - 1;                                 // tail: same bytes, same place as the last token
        orow[k] = reinterpret_cast<char*>(reinterpret_cast<OT*>(const_cast<void*>(a.x)) + (tr.x_row0 + t) * a.ld_x) +
                  (lane % OS::COLS) * 16;
    }
    // mu sits in LDS behind the ring: a global load inside the loop would make the compiler
    // wait for everything in flight, the asynchronous transfers included
    float* mu_lds = reinterpret_cast<float*>(smem + NSTAGE * SLAB_U4);
    for (int i = tid; i < p; i += kThreads) mu_lds[i] = P->mu[i];
    const float* mu = mu_lds + 16 * h;
    char* ostage = reinterpret_cast<char*>(mu_lds + p) + wave * (TOK_W * OS::ROW_B);       // this wave's transpose tile

#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < n_ft) issue(u, u);
    wait_vmem_times<NV>(min(D - 1, n_ft - 1));
    __syncthreads();

    auto tile_step = [&](int ft, int stage) {
        if (ft + D < n_ft) issue(ft + D, (stage + D) % NSTAGE);
        f32x16 acc[TT];
        {
            f32x16 m;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = *reinterpret_cast<const float4*>(mu + ft * 32 + 4 * q);
                m[4 * q] = v.x; m[4 * q + 1] = v.y; m[4 * q + 2] = v.z; m[4 * q + 3] = v.w;
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[tt] = m;
        }
        constexpr int NSTEP = 2 * NCT;
        const uint4* abase = smem + stage * SLAB_U4 + lane;
        uint4 af[3];
        af[0] = abase[0];
        af[1] = abase[64];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < NSTEP; ++ks) {
            if (ks + 2 < NSTEP) af[(ks + 2) % 3] = abase[(ks + 2) * 64];
            const bf16x8 av = as_bf16x8_d(af[ks % 3]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bop[tt][ks], acc[tt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) stage_put(ostage, tt * 32 + l32, h, ft % OS::FT_PER_ROW, acc[tt], OT());
        // the slab of the next step (issued at the top of this one) must have landed; everything
        // older -- the previous stores included -- is then complete as well (issue-order completion)
        wait_vmem<0>();
        __syncthreads();
        if (ft % OS::FT_PER_ROW == OS::FT_PER_ROW - 1) {
            // the 128-byte rows are complete: read them back row-contiguous (the
            // barrier also orders this wave's LDS writes before these reads) and store whole lines
            uint4 o[NS];
#pragma unroll
            for (int k = 0; k < NS; ++k)
                o[k] = *reinterpret_cast<const uint4*>(ostage + srow[k] * OS::ROW_B + (((lane % OS::COLS) ^ OS::swz(srow[k])) * 16));
#pragma unroll
            for (int k = 0; k < NS; ++k) *reinterpret_cast<uint4*>(orow[k] + (size_t)(ft / OS::FT_PER_ROW) * OS::ROW_B) = o[k];
        }
    };
    for (int f0 = 0; f0 < n_ft; f0 += NSTAGE) {
#pragma unroll
        for (int u = 0; u < NSTAGE; ++u)
            if (f0 + u < n_ft) tile_step(f0 + u, u);
    }
    __syncthreads();
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
    const int slab_b = 2 * 2 * nct * 1024 + p * 4 + tok_wg * 128;
    (void)dtype;
    return rec_b > slab_b ? rec_b : slab_b;
}

}  // namespace kvtc
