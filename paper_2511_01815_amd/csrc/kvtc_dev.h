// Device-side descriptors and the job -> tile scheduling shared by the encode and
// decode kernels.  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <mutex>
#include <utility>
#include <vector>
#include "../../include/kvtc.h"

namespace kvtc {

constexpr int kThreads = 256;          // 4 wavefronts, one per SIMD of a compute unit
constexpr int kMaxJobs = 1024;         // jobs per batched launch (tile table lives in LDS)
constexpr int kLdsBudget = 160 * 1024; // gfx950 LDS per workgroup
constexpr int kJobTableBytes = (kMaxJobs + 1) * 4;
constexpr int kEncShortTile = 64;      // tokens per workgroup tile of the encode variants for short jobs
constexpr int kDecShortTile = 128;     // the same for decode (one token tile per wave)

// Lets a kernel use the whole LDS of a compute unit as dynamic shared memory.  The attribute
// sticks to the (device, function) pair, so it is set on the first launch there only.
inline hipError_t allow_full_lds(const void* fn) {
    static std::mutex m;
    static std::vector<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(m);
    for (const auto& d : done)
        if (d.first == dev && d.second == fn) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
    if (e == hipSuccess) done.emplace_back(dev, fn);
    return e;
}

// Everything a kernel needs to know about a plan.  Lives in device memory and is read
// through wave-uniform (scalar) loads.
struct PlanDev {
    int32_t p, r, n_groups, n_blocks;       // n_blocks = r / 16
    int32_t rec_dwords;                     // R / 4
    int32_t enc_ntw, enc_wc;                // encode variant: coefficient tiles per wave, waves across coefficients
    int32_t dec_nct, dec_tt;                // decode variant: coefficient tiles, token tiles per wave
    int32_t enc_tok_wg, dec_tok_wg;         // tokens per workgroup tile
    int32_t enc_lds[2];                     // encode: dynamic LDS bytes needed (without the job table), per element dtype
    int32_t dec_rec_lds, dec_ring_lds;      // decode: bytes of the record image, of the basis ring + mu
    int32_t code_bits_max;                  // widest code of the plan
    int32_t enc_wgs, dec_wgs;               // workgroups per compute unit the variant is built for (1..3)
    int32_t enc_nw, enc_s_key;              // encode: waves per workgroup (4 or 8); key of the variant for short jobs (64-token tiles), 0 = none
    int32_t dec_cls, reserved0;             // decode: the kernel class that serves the plan = the widest plan of the class, in coordinate tiles (dec_nct: the width the plan runs at, one of those built for the class)
    const uint4* v_enc;    // [p/16][32*ntp/32][64] MFMA A fragments of V_kept^T (encode)
    const uint4* v_dec;    // [p/32][2*nct*64 + 16] MFMA B fragments of V_kept^T (decode), then the tile's 32 mu entries; tiles 2k, 2k+1 = even, odd features of span k
    const float* negc;     // [32*ntp]  -(mu^T V_kept), zero in the padding
    const float* mu;       // [p]
    const uint32_t* blk;   // [64] per 16-coordinate block: bits | group << 8 | halfword offset << 16; 0 = padding
    const uint32_t* grp;   // [n_groups] first block | n blocks << 8 | bits << 16
};

struct KernelArgs {
    const PlanDev* plans;      // device array
    int32_t n_plans;
    const kvtc_job* jobs;      // device array, or nullptr -> `single`
    int32_t n_jobs;
    kvtc_job single;
    const uint64_t* offsets;   // device, [n_jobs + 1], or nullptr (single job at offset 0)
    const void* x;             // feature array (encode: input, decode: output)
    int64_t ld_x;
    int32_t x_blk_log2;        // 0: a token's features are contiguous.  Else they come in blocks of 2^x_blk_log2 features (a head, a layer) ...
    int64_t x_blk_jump;        // ... and x_blk_jump elements lie between the end of a block and the start of the token's next one
    void* stream_buf;          // record stream (encode: output, decode: input)
    uint64_t cap;              // bytes available in stream_buf
    uint32_t* status;          // device, may be nullptr
    uint32_t dec_ring_off;     // decode: byte offset of the basis ring in the work area; 0 = it shares the record image's space
    int32_t enc_short;         // encode: this launch runs the short-job variants (jobs of at most enc_short_max tokens whose plan has one) ...
    int32_t enc_short_max;     // ... and the launches of the bulk variants leave those jobs alone; 0 = no job counts as short
    int32_t dec_short;         // decode: this launch runs the one-token-tile-per-wave variant of every plan (128-token tiles)
    int32_t dec_accumulate;    // decode of a sectioned plan: 1 = fp32 output, add the product to the output instead of storing it (a further section);
                               // 2 = bf16 output, store round(dec_sum + product) (the last section)
    const float* dec_sum;      // mode 2: the earlier sections' fp32 sums, [tokens][dec_sum_ld], features contiguous
    int64_t dec_sum_ld;
};

struct TileRef {
    int32_t job, plan, n_tokens;
    int64_t x_row0;
    uint64_t offset;
    int32_t tile;      // tile index inside the job
};

// Builds the exclusive prefix of tiles per job in LDS (tile_start[0..n_jobs]) and returns
// the total.  A job with a bad plan index, a negative token count or a stream that would end
// beyond `cap` gets zero tiles, and so does a job whose plan belongs to another kernel variant
// (variant_key: the variant's parameters in decimal positions); workgroup 0 reports the lowest bad job in *status.
template <bool kEncode, int NT = kThreads>
__device__ inline uint32_t build_tile_table(const KernelArgs& a, int variant_key, uint32_t* tile_start, uint32_t* scratch /*[NT + 1]*/) {
    const int tid = threadIdx.x;
    const int n_jobs = a.jobs ? a.n_jobs : 1;
    const int per = (n_jobs + NT - 1) / NT;
    const int j0 = tid * per;
    uint32_t local[kMaxJobs / NT];
    uint32_t sum = 0;
    uint32_t first_bad = 0xffffffffu;
#pragma unroll
    for (int k = 0; k < kMaxJobs / NT; ++k) {
        uint32_t tiles = 0;
        const int j = j0 + k;
        if (k < per && j < n_jobs) {
            const kvtc_job jb = a.jobs ? a.jobs[j] : a.single;
            bool ok = jb.plan >= 0 && jb.plan < a.n_plans && jb.n_tokens >= 0;
            if (ok && a.offsets) {
                // the job's own extent must lie inside the buffer (offsets need not be a running sum:
                // an append writes each job into its own region)
                const uint64_t off = a.offsets[j], bytes = (uint64_t)jb.n_tokens * (uint64_t)a.plans[jb.plan].rec_dwords * 4ull;
                ok = off <= a.cap && bytes <= a.cap - off;
            }
            if (ok) {
                const PlanDev& pl = a.plans[jb.plan];
                // each launch serves the plans of its own kernel variant; other launches take the rest.
                // Encode: short jobs go to the plan's short-job variant (narrow tiles), if it has one.
                const bool is_short = kEncode && pl.enc_s_key != 0 && jb.n_tokens <= a.enc_short_max;
                int tw = kEncode ? pl.enc_tok_wg : pl.dec_tok_wg;
                int key = kEncode ? pl.enc_nw * 10000 + pl.enc_wc * 100 + pl.enc_ntw : pl.dec_tt * 100 + pl.dec_cls;
                if (!kEncode && a.dec_short) { tw = kDecShortTile; key = 100 + pl.dec_cls; }
                if (kEncode && a.enc_short) { tw = kEncShortTile; key = is_short ? pl.enc_s_key : -1; }
                else if (is_short) key = -1;
                if (key == variant_key) tiles = (uint32_t)((jb.n_tokens + tw - 1) / tw);
            } else if (first_bad == 0xffffffffu) {
                first_bad = (uint32_t)j;
            }
        }
        local[k] = tiles;
        sum += tiles;
    }
    // exclusive scan of the per-thread sums
    scratch[tid] = sum;
    __syncthreads();
    for (int d = 1; d < NT; d <<= 1) {
        uint32_t v = tid >= d ? scratch[tid - d] : 0u;
        __syncthreads();
        scratch[tid] += v;
        __syncthreads();
    }
    uint32_t run = scratch[tid] - sum;
    const uint32_t total = scratch[NT - 1];
#pragma unroll
    for (int k = 0; k < kMaxJobs / NT; ++k) {
        const int j = j0 + k;
        if (k < per && j < n_jobs) tile_start[j] = run;
        run += local[k];
    }
    if (tid == 0) tile_start[n_jobs] = total;
    __syncthreads();
    // lowest bad job -> status (workgroup 0 only; a plain vector store)
    if (a.status && blockIdx.x == 0) {
        scratch[tid] = first_bad;
        __syncthreads();
        for (int d = NT / 2; d > 0; d >>= 1) {
            if (tid < d) scratch[tid] = min(scratch[tid], scratch[tid + d]);
            __syncthreads();
        }
        if (tid == 0 && scratch[0] != 0xffffffffu) *a.status = scratch[0] + 1u;
    }
    __syncthreads();
    return total;
}

// A pointer whose value is the same in every lane, moved into scalar registers.
template <typename T> __device__ __forceinline__ const T* uniform_ptr(const T* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}

// Wave-uniform loads through the scalar unit (read-only data written before the launch: job
// list, stream offsets, plan descriptors).  They count on lgkmcnt, not on vmcnt, so they neither
// wait for nor disturb the vector-memory operations a kernel keeps in flight.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 sload_x4(const void* p_uniform) {
    u32x4 v;
    asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_ptr(reinterpret_cast<const char*>(p_uniform))) : "memory");
    return v;
}
__device__ __forceinline__ u32x2 sload_x2(const void* p_uniform) {
    u32x2 v;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_ptr(reinterpret_cast<const char*>(p_uniform))) : "memory");
    return v;
}
template <typename T> __device__ __forceinline__ T* sload_ptr(const void* p_uniform) {
    const u32x2 v = sload_x2(p_uniform);
    return reinterpret_cast<T*>(((uint64_t)v[1] << 32) | v[0]);
}

// The fields of a plan descriptor the decode kernel uses, in scalar registers.
struct PlanDec {
    int32_t p, rec_dwords, dec_nct, dec_tt, dec_tok_wg, code_bits_max;
    const uint4* v_dec;
    const uint32_t* blk;
};
__device__ __forceinline__ PlanDec load_plan_dec(const PlanDev* P) {
    static_assert(offsetof(PlanDev, p) == 0 && offsetof(PlanDev, rec_dwords) == 16 && offsetof(PlanDev, dec_nct) == 28 &&
                  offsetof(PlanDev, dec_tt) == 32 && offsetof(PlanDev, dec_tok_wg) == 40, "descriptor layout");
    const char* b = reinterpret_cast<const char*>(P);
    static_assert(offsetof(PlanDev, code_bits_max) == 60, "descriptor layout");
    const u32x4 q0 = sload_x4(b), q1 = sload_x4(b + 16), q2 = sload_x4(b + 32), q3 = sload_x4(b + 48);
    PlanDec d;
    d.p = (int32_t)q0[0];
    d.rec_dwords = (int32_t)q1[0];
    d.dec_nct = (int32_t)q1[3];
    d.dec_tt = (int32_t)q2[0];
    d.dec_tok_wg = (int32_t)q2[2];
    d.code_bits_max = (int32_t)q3[3];
    d.v_dec = sload_ptr<const uint4>(b + offsetof(PlanDev, v_dec));
    d.blk = sload_ptr<const uint32_t>(b + offsetof(PlanDev, blk));
    return d;
}

// The fields of a plan descriptor the encode kernel uses, in scalar registers.
struct PlanEnc {
    int32_t p, n_groups, rec_dwords, enc_ntw, enc_wc, code_bits_max;
    const uint4* v_enc;
    const float* negc;
    const uint32_t* blk;
    const uint32_t* grp;
};
__device__ __forceinline__ PlanEnc load_plan_enc(const PlanDev* P) {
    static_assert(offsetof(PlanDev, n_groups) == 8 && offsetof(PlanDev, enc_ntw) == 20 && offsetof(PlanDev, enc_wc) == 24, "descriptor layout");
    const char* b = reinterpret_cast<const char*>(P);
    const u32x4 q0 = sload_x4(b), q1 = sload_x4(b + 16), q3 = sload_x4(b + 48);
    PlanEnc d;
    d.code_bits_max = (int32_t)q3[3];
    d.p = (int32_t)q0[0];
    d.n_groups = (int32_t)q0[2];
    d.rec_dwords = (int32_t)q1[0];
    d.enc_ntw = (int32_t)q1[1];
    d.enc_wc = (int32_t)q1[2];
    d.v_enc = sload_ptr<const uint4>(b + offsetof(PlanDev, v_enc));
    d.negc = sload_ptr<const float>(b + offsetof(PlanDev, negc));
    d.blk = sload_ptr<const uint32_t>(b + offsetof(PlanDev, blk));
    d.grp = sload_ptr<const uint32_t>(b + offsetof(PlanDev, grp));
    return d;
}

// The tiles of a persistent workgroup: first, first + step, ... below end.  Workgroups are dealt to the
// chip's eight XCDs round-robin (workgroup b runs on XCD b % 8; read back from the hardware's XCC id), and
// each XCD has an L2 of its own.  Every round of gridDim tiles is therefore cut into eight contiguous blocks,
// one per XCD: the workgroups of an XCD then work on the same tensor (or two) at any time and touch one
// basis, not the four that a round spans -- with a basis per tensor the decode of the 32-layer cache
// measured 6 % faster this way (its basis slabs compete for the L2 with 4 GiB of output passing through);
// the whole launch still sweeps memory as one window.  (Wherever the hardware places a workgroup, every
// tile is done exactly once.)
struct TileRange { uint32_t first, end, step; };
__device__ __forceinline__ TileRange my_tiles(uint32_t total) {
    const uint32_t g = gridDim.x, b = blockIdx.x;
    if ((g & 7u) != 0u || total < 2u * g) return TileRange{b, total, g};
    return TileRange{(b & 7u) * (g >> 3) + (b >> 3), total, g};
}

__device__ inline TileRef find_tile(const KernelArgs& a, const uint32_t* tile_start, uint32_t tile) {
    const int n_jobs = a.jobs ? a.n_jobs : 1;
    int lo = 0, hi = n_jobs;                 // invariant: tile_start[lo] <= tile < tile_start[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_start[mid] <= tile) lo = mid; else hi = mid;
    }
    lo = __builtin_amdgcn_readfirstlane(lo);
    static_assert(sizeof(kvtc_job) == 16 && offsetof(kvtc_job, n_tokens) == 4 && offsetof(kvtc_job, x_row0) == 8, "job layout");
    TileRef t;
    t.job = lo;
    if (a.jobs) {
        const u32x4 jb = sload_x4(a.jobs + lo);
        t.plan = (int32_t)jb[0];
        t.n_tokens = (int32_t)jb[1];
        t.x_row0 = (int64_t)(((uint64_t)jb[3] << 32) | jb[2]);
    } else {
        t.plan = a.single.plan;
        t.n_tokens = a.single.n_tokens;
        t.x_row0 = a.single.x_row0;
    }
    t.offset = 0ull;
    if (a.offsets) {
        const u32x2 o = sload_x2(a.offsets + lo);
        t.offset = ((uint64_t)o[1] << 32) | o[0];
    }
    t.tile = (int32_t)(tile - tile_start[lo]);
    t.tile = __builtin_amdgcn_readfirstlane(t.tile);
    return t;
}

// LDS byte offset of a pointer into shared memory.
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(size_t)(const __attribute__((address_space(3))) void*)p;
}

// 16 bytes per lane from global memory straight into LDS, no register staging: lane i's bytes
// land at lds_byte_addr + 16 * i (wave-uniform address; it goes through M0).  Issued behind the
// compiler's back: the compiler neither orders later LDS reads after it nor counts it, so a
// step's transfers can stay in flight while the previous slab is read (the builtin form makes the
// compiler wait for vmcnt(0) before any later LDS read).  The caller owns the wait: wait_vmem<N>()
// before the barrier that publishes the data.
__device__ __forceinline__ void dma16_async(const void* gsrc, uint32_t lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gsrc), "s"(lds_byte_addr) : "memory");
}

// The same with a wave-uniform base (scalar registers) plus a 32-bit per-lane byte offset: the
// per-transfer address arithmetic stays on the scalar unit and costs no vector registers.
// (Values the compiler cannot prove uniform would reach the "s" operands in vector registers, so
// both go through readfirstlane, which folds away when they already are scalar.)
__device__ __forceinline__ void dma16_async(const void* base_uniform, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane_byte_off), "s"(uniform_ptr(reinterpret_cast<const char*>(base_uniform))),
                    "s"(__builtin_amdgcn_readfirstlane(lds_byte_addr)) : "memory");
}

// One dword per lane: lane i's dword lands at lds_byte_addr + 4 * i.
__device__ __forceinline__ void dma4_async(const void* base_uniform, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(lane_byte_off), "s"(uniform_ptr(reinterpret_cast<const char*>(base_uniform))),
                    "s"(__builtin_amdgcn_readfirstlane(lds_byte_addr)) : "memory");
}

// s_waitcnt vmcnt(N) only (N <= 63): the N most recent vector-memory operations may stay in flight.
template <int N> __device__ __forceinline__ void wait_vmem() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// s_waitcnt vmcnt(n) with a wave-uniform run-time n; n above 63 waits as for 63.
__device__ __forceinline__ void wait_vmem_dyn(int n) {
#define KVTC_W(N) case N: wait_vmem<N>(); break;
#define KVTC_W8(N) KVTC_W(N) KVTC_W(N + 1) KVTC_W(N + 2) KVTC_W(N + 3) KVTC_W(N + 4) KVTC_W(N + 5) KVTC_W(N + 6) KVTC_W(N + 7)
    switch (n < 0 ? 0 : (n > 63 ? 63 : n)) {
        KVTC_W8(0) KVTC_W8(8) KVTC_W8(16) KVTC_W8(24) KVTC_W8(32) KVTC_W8(40) KVTC_W8(48) KVTC_W8(56)
    }
#undef KVTC_W8
#undef KVTC_W
}
// Wait until at most k * N operations are in flight, k in 0..3 chosen at run time (wave-uniform).
template <int N> __device__ __forceinline__ void wait_vmem_times(int k) {
    if (k <= 0) wait_vmem<0>();
    else if (k == 1) wait_vmem<N>();
    else if (k == 2) wait_vmem<2 * N>();
    else wait_vmem<3 * N>();
}

}  // namespace kvtc
