// Host side of the C ABI declared in include/kvtc.h: argument checks, plan compilation
// (swizzling the basis into matrix-core operand fragments, block/group tables), launches,
// and the on-device prefix sum of stream offsets.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kvtc_dev.h"
#include "kvtc_numeric.h"
#include "../../include/kvtc_test_hooks.h"

namespace kvtc {
hipError_t launch_encode(const KernelArgs& a, kvtc_dtype dtype, int key, int grid, size_t lds_bytes, hipStream_t stream);
hipError_t launch_decode(const KernelArgs& a, kvtc_dtype dtype, int key, int grid, size_t lds_bytes, hipStream_t stream);
int encode_lds_bytes(int ntw, int wc, int nw, int n_groups, int rec_dwords, kvtc_dtype dtype);
int encode_tok_wg(int ntw, int wc, int nw);
hipError_t launch_fp8_pack(const void* x, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld_x, void* out, hipStream_t stream);
hipError_t launch_fp8_unpack(const void* in, int64_t n_tokens, int p, void* x, kvtc_dtype dtype, int64_t ld_x, hipStream_t stream);
hipError_t launch_offsets_append(const uint32_t* rec_dwords, int n_plans, const kvtc_job* jobs, int n_jobs, const uint64_t* region,
                                 const int64_t* n_coded, uint64_t* offsets, hipStream_t stream);
struct RopeArgs {
    void* x;
    int64_t n_tokens, token_stride, head_stride;
    const int32_t* positions;
    int64_t position0;
    int32_t n_heads, d_head, inverse;
    double theta[128];
};
hipError_t launch_rope(const RopeArgs& a, kvtc_dtype dtype, int interleaved, int grid, hipStream_t stream);
hipError_t launch_calib_moments(const void* x, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld, int blk_log2, int64_t blk_jump,
                                double* sum, double* gram, hipStream_t stream);
int decode_rec_bytes(int tt, int rec_dwords);
int decode_ring_bytes(int nct);
int decode_stage_u4(int nct);
}  // namespace kvtc

using namespace kvtc;

struct kvtc_plan {
    PlanDev h;              // host copy of the descriptor (device pointers inside)
    void* blob;             // one device allocation holding everything
    PlanDev* desc_dev;      // the descriptor inside the blob
    size_t record_bytes;
    int enc_s_wgs;          // short-job encode variant (key in h.enc_s_key, 0 = none): workgroups per compute unit ...
    int enc_s_lds[2];       // ... and dynamic LDS bytes per element dtype
};

struct kvtc_batch {
    PlanDev* plans_dev;
    int n_plans;
    // the kernel variants the plans use (a launch per variant), with the LDS maxima over each one's plans
    struct EncVariant { int key, wgs, lds[2]; };        // workgroups per compute unit; lds per element dtype
    struct DecVariant { int key, wgs, rec, ring; };     // workgroups per compute unit; record image, basis ring (the widest among the class's plans)
    std::vector<EncVariant> enc;
    std::vector<EncVariant> enc_short;                  // the short-job variants among the plans (64-token tiles)
    std::vector<DecVariant> dec;
    int max_p;
    std::vector<int32_t> ps;                            // the distinct feature counts among the plans
    std::vector<int32_t> rec_dwords;
    uint32_t* rec_dwords_dev;
};

namespace {

thread_local char g_err[256] = "";

kvtc_status fail(kvtc_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

float bf16_bits_to_float(uint16_t b) { return bits_f32((uint32_t)b << 16); }

// Compute units of the current device (cached per device).
int cu_count() {
    static int n[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (n[dev] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) n[dev] = prop.multiProcessorCount;
        if (n[dev] <= 0) n[dev] = 256;
    }
    return n[dev];
}

// Row pitch limit (elements): the kernels address a workgroup tile of up to 256 rows with 32-bit byte offsets.
constexpr int kMaxPitch = 1 << 21;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// position of coordinate/feature row `rho` of an MFMA tile inside the lane's 16 results:
// the 32x32 accumulator gives lane half hh, register i the row 8*(i/4) + 4*hh + i%4; mapping
// row rho to index 16*hh + i makes each lane own 16 consecutive indices.
int permuted_index(int rho) {
    const int q = rho >> 3, hh = (rho >> 2) & 1, m = rho & 3;
    return 16 * hh + 4 * q + m;
}

bool dtype_ok(kvtc_dtype d) { return d == KVTC_BF16 || d == KVTC_F32; }
size_t elem_size(kvtc_dtype d) { return d == KVTC_BF16 ? 2 : 4; }

__global__ void __launch_bounds__(256) offsets_kernel(const uint32_t* rec_dwords, int n_plans, const kvtc_job* jobs,
                                                     int n_jobs, uint64_t* offsets, uint64_t* offsets_copy /*may be null*/) {
    __shared__ uint64_t s[256];
    __shared__ uint64_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n_jobs; base += 256) {
        const int j = base + tid;
        uint64_t bytes = 0;
        if (j < n_jobs) {
            const kvtc_job jb = jobs[j];
            if (jb.plan >= 0 && jb.plan < n_plans && jb.n_tokens > 0)
                bytes = (uint64_t)jb.n_tokens * rec_dwords[jb.plan] * 4ull;
        }
        s[tid] = bytes;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const uint64_t v = tid >= d ? s[tid - d] : 0ull;
            __syncthreads();
            s[tid] += v;
            __syncthreads();
        }
        const uint64_t c = carry;
        if (j < n_jobs) {
            offsets[j] = c + s[tid] - bytes;
            if (offsets_copy) offsets_copy[j] = c + s[tid] - bytes;
        }
        __syncthreads();
        if (tid == 255) carry = c + s[255];
        __syncthreads();
    }
    if (tid == 0) {
        offsets[n_jobs] = carry;
        if (offsets_copy) offsets_copy[n_jobs] = carry;
    }
}

// ---- the entry point that allocates nothing ------------------------------------------------------
// Its plan-descriptor table, record-size table and stream offsets -- what kvtc_batch_create and the
// caller's offsets buffer hold for kvtc_encode_batch -- live in this file-scope device array.  Every
// GPU the library runs on holds its own copy (about 17 KB) until the process ends.  The name is a
// host-side stand-in, not a device address: host code only ever uses the per-device pointer that
// hipGetSymbolAddress returned for it.
constexpr int kStaticMaxPlans = 64;
struct StaticScratch {
    PlanDev plans[kStaticMaxPlans];
    uint32_t rec_dwords[kStaticMaxPlans];
    uint64_t offsets[kMaxJobs + 1];
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];

struct PlanPtrs { const PlanDev* p[kStaticMaxPlans]; };

// descriptor of plan i (inside the plan's own device blob) -> table entry i; one thread per dword
__global__ void __launch_bounds__(256) gather_plans_kernel(const PlanPtrs src, int n_plans, StaticScratch* sc) {
    constexpr int kDw = (int)(sizeof(PlanDev) / 4);
    static_assert(sizeof(PlanDev) % 4 == 0, "descriptor is whole dwords");
    for (int i = threadIdx.x; i < n_plans * kDw; i += blockDim.x) {
        const int pl = i / kDw, w = i - pl * kDw;
        reinterpret_cast<uint32_t*>(&sc->plans[pl])[w] = reinterpret_cast<const uint32_t*>(src.p[pl])[w];
    }
    for (int i = threadIdx.x; i < n_plans; i += blockDim.x) sc->rec_dwords[i] = (uint32_t)src.p[i]->rec_dwords;
}

// per-device address of `scratch`, looked up once per device with that device current
hipError_t static_scratch(StaticScratch** out) {
    static std::mutex m;
    static StaticScratch* ptr[64] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(m);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        ptr[dev] = static_cast<StaticScratch*>(p);
    }
    *out = ptr[dev];
    return hipSuccess;
}

// Decode LDS layout for one launch: record image and basis ring side by side when both fit (narrow
// variants: within their share of a compute unit's LDS, so that all their workgroups stay resident), which lets each
// tile's records be fetched during the previous tile's sweep; otherwise they share the space.
struct DecLayout { uint32_t ring_off; size_t lds_bytes; };
DecLayout decode_layout(int rec_b, int ring_b, int wgs_per_cu) {
    const int budget = kLdsBudget / wgs_per_cu - kJobTableBytes - 64;
    if (rec_b + ring_b <= budget) return {(uint32_t)rec_b, (size_t)kJobTableBytes + 64 + rec_b + ring_b};
    return {0u, (size_t)kJobTableBytes + 64 + (rec_b > ring_b ? rec_b : ring_b)};
}

}  // namespace

namespace kvtc {
// for the library's other sources: records the message kvtc_last_error returns on this thread
kvtc_status set_error(kvtc_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}
}  // namespace kvtc

extern "C" {

const char* kvtc_last_error(void) { return g_err; }

uint16_t kvtc_host_f16_round_down(float x) { return f16_round_dir(x, false); }
uint16_t kvtc_host_f16_round_up(float x) { return f16_round_dir(x, true); }
void kvtc_host_group_header(float lo, float hi, int bits, uint16_t* shift16, uint16_t* scale16) {
    const GroupQ q = group_header(lo, hi, bits);
    if (shift16) *shift16 = q.shift16;
    if (scale16) *scale16 = q.scale16;
}
uint32_t kvtc_host_code(float d, uint16_t shift16, uint16_t scale16, int bits) {
    const float sc = f16_bits_to_f32(scale16);
    const float inv = sc > 0.0f ? div_rn(1.0f, sc) : 0.0f;          // as group_header derives it
    return (uint32_t)code_of(d, f16_bits_to_f32(shift16), inv, (float)((1u << bits) - 1u));
}

// v_kept_host: [p] rows of ldv elements, of which the first r are the plan's columns.  dec_zero_mu: the decode side adds
// no mean (a further section of a sectioned plan: the first section's decode has added it already).
static kvtc_status plan_create_impl(kvtc_plan** out, int p, int r, const float* mu_host, const uint16_t* v_kept_host, size_t ldv,
                                    int n_groups, const kvtc_group* groups_host, bool dec_zero_mu, kvtc_stream stream);

kvtc_status kvtc_plan_create(kvtc_plan** out, int p, int r, const float* mu_host, const uint16_t* v_kept_host,
                             int n_groups, const kvtc_group* groups_host, kvtc_stream stream) {
    return plan_create_impl(out, p, r, mu_host, v_kept_host, (size_t)(r > 0 ? r : 0), n_groups, groups_host, false, stream);
}

static kvtc_status plan_create_impl(kvtc_plan** out, int p, int r, const float* mu_host, const uint16_t* v_kept_host, size_t ldv,
                                    int n_groups, const kvtc_group* groups_host, bool dec_zero_mu, kvtc_stream stream) {
    if (out) *out = nullptr;
    if (!out || !mu_host || !v_kept_host || !groups_host) return fail(KVTC_E_ARG, "kvtc_plan_create: null argument");
    if (p <= 0 || p % 64 != 0) return fail(KVTC_E_ARG, "kvtc_plan_create: p=%d must be a positive multiple of 64", p);
    if (r < 16 || r > 1024) return fail(KVTC_E_ARG, "kvtc_plan_create: r=%d outside 16..1024", r);
    if (n_groups < 1 || n_groups > 64) return fail(KVTC_E_ARG, "kvtc_plan_create: n_groups=%d outside 1..64", n_groups);
    long sum = 0, payload_bits = 0;
    for (int g = 0; g < n_groups; ++g) {
        if (groups_host[g].n < 1) return fail(KVTC_E_ARG, "kvtc_plan_create: group %d is empty", g);
        if (groups_host[g].bits < 1 || groups_host[g].bits > 16)
            return fail(KVTC_E_ARG, "kvtc_plan_create: group %d has %d bits (1..16 allowed)", g, groups_host[g].bits);
        sum += groups_host[g].n;
        payload_bits += (long)groups_host[g].n * groups_host[g].bits;
    }
    if (sum != r) return fail(KVTC_E_ARG, "kvtc_plan_create: group sizes sum to %ld, r=%d", sum, r);
    for (int g = 0; g < n_groups; ++g)
        if (groups_host[g].n % 16 != 0)
            return fail(KVTC_E_UNSUPPORTED, "kvtc_plan_create: group %d has %d coordinates; the kernels need multiples of 16",
                        g, groups_host[g].n);

    PlanDev d;
    memset(&d, 0, sizeof(d));
    d.p = p;
    d.r = r;
    d.n_groups = n_groups;
    d.n_blocks = r / 16;
    for (int g = 0; g < n_groups; ++g)
        if (groups_host[g].bits > d.code_bits_max) d.code_bits_max = groups_host[g].bits;
    const long total_bits = 32L * n_groups + payload_bits;
    d.rec_dwords = (int)((total_bits + 31) / 32);
    const int nt = (r + 31) / 32;

    // encode variant: NTW coordinate tiles per wave, WC waves across coordinates, NW waves per workgroup.
    // Up to 320 padded coordinates a 4-wave workgroup keeps its tile (64 tokens per wave across the
    // tokens; 96 in the 8-tile variant) x all its coordinates in 256 registers per lane and two
    // workgroups share a compute unit (three where 168 registers suffice: measured 5 % faster on the
    // 6-tile encode).  From 321 to 640, 8-wave workgroups (two waves per SIMD at 256 registers,
    // 128-token tiles, four waves across the coordinates) measured twice as fast as 4-wave ones with
    // 512 registers; beyond that only the latter hold a tile.
    // {waves across coordinates, tiles per wave, workgroups per compute unit, waves per workgroup}, ascending padded width
    static const int enc_tab[][4] = {{1, 2, 2, 4}, {1, 4, 2, 4}, {2, 3, 3, 4}, {2, 4, 2, 4}, {2, 5, 2, 4},
                                     {4, 3, 1, 8}, {4, 4, 1, 8}, {4, 5, 1, 8}, {4, 6, 1, 4}, {4, 8, 1, 4}};
    d.enc_wc = 0;
    for (auto& e : enc_tab)
        if (e[0] * e[1] >= nt) { d.enc_wc = e[0]; d.enc_ntw = e[1]; d.enc_wgs = e[2]; d.enc_nw = e[3]; break; }
    // decode: the widths the kernels are built for, with the register class (= its widest member) that serves each;
    // odd widths where the calibrated plans of the 8B-shaped cache fall (224 = 7, 272 = 9, 528 = 17 tiles): in decode
    // the coordinates are the contraction index, so a tile less is that much less matrix work and basis traffic
    // {token tiles per wave, coordinate tiles, class, workgroups per compute unit}
    static const int dec_tab[][4] = {{2, 2, 4, 3}, {2, 4, 4, 3}, {2, 6, 10, 2}, {2, 7, 10, 2}, {2, 8, 10, 2}, {2, 9, 10, 2}, {2, 10, 10, 2},
                                     {2, 12, 18, 1}, {2, 16, 18, 1}, {2, 17, 18, 1}, {2, 18, 18, 1}, {2, 20, 24, 1}, {2, 24, 24, 1}, {1, 32, 32, 1}};
    d.dec_tt = 0;
    for (auto& e : dec_tab)
        if (e[1] >= nt) { d.dec_tt = e[0]; d.dec_nct = e[1]; d.dec_cls = e[2]; d.dec_wgs = e[3]; break; }
    if (d.enc_wc == 0 || d.dec_tt == 0) return fail(KVTC_E_UNSUPPORTED, "kvtc_plan_create: no kernel variant for r=%d", r);
    const int ntp = d.enc_ntw * d.enc_wc;
    d.enc_tok_wg = encode_tok_wg(d.enc_ntw, d.enc_wc, d.enc_nw);
    d.dec_tok_wg = 4 * 32 * d.dec_tt;
    {
        d.enc_lds[KVTC_BF16] = encode_lds_bytes(d.enc_ntw, d.enc_wc, d.enc_nw, n_groups, d.rec_dwords, KVTC_BF16);
        d.enc_lds[KVTC_F32] = encode_lds_bytes(d.enc_ntw, d.enc_wc, d.enc_nw, n_groups, d.rec_dwords, KVTC_F32);
        d.dec_rec_lds = decode_rec_bytes(d.dec_tt, d.rec_dwords);
        d.dec_ring_lds = decode_ring_bytes(d.dec_nct);
    }
    const int lds_cap = kLdsBudget - kJobTableBytes - 64;
    const int dec_need = d.dec_rec_lds > d.dec_ring_lds ? d.dec_rec_lds : d.dec_ring_lds;
    if (d.enc_lds[0] > lds_cap || d.enc_lds[1] > lds_cap || dec_need > lds_cap)
        return fail(KVTC_E_UNSUPPORTED,
                    "kvtc_plan_create: record of %d bytes with r=%d needs %d/%d/%d bytes of LDS, %d available",
                    d.rec_dwords * 4, r, d.enc_lds[0], d.enc_lds[1], dec_need, lds_cap);

    // encode variant for short jobs: the same padded width with one wave across the tokens (64-token tiles);
    // the two widest bulk variants already are of that shape
    // {padded tiles, waves across coordinates, tiles per wave, waves per workgroup}
    static const int enc_short_tab[][4] = {{2, 2, 1, 2}, {4, 4, 1, 4}, {6, 2, 3, 2}, {8, 4, 2, 4}, {10, 2, 5, 2},
                                           {12, 4, 3, 4}, {16, 4, 4, 4}, {20, 4, 5, 4}};
    d.enc_s_key = 0;
    int s_wgs = 1, s_lds[2] = {0, 0};
    for (auto& e : enc_short_tab)
        if (e[0] == ntp && encode_tok_wg(e[2], e[1], e[3]) == kEncShortTile) {
            s_lds[KVTC_BF16] = encode_lds_bytes(e[2], e[1], e[3], n_groups, d.rec_dwords, KVTC_BF16);
            s_lds[KVTC_F32] = encode_lds_bytes(e[2], e[1], e[3], n_groups, d.rec_dwords, KVTC_F32);
            if (s_lds[0] <= lds_cap && s_lds[1] <= lds_cap) {
                d.enc_s_key = e[3] * 10000 + e[1] * 100 + e[2];
                s_wgs = e[3] == 4 && ntp <= 10 ? 2 : 1;          // as the kernel's launch bounds
            }
        }

    // ---- host images ---------------------------------------------------------------
    const size_t n_venc = (size_t)(p / 16) * ntp * 64 * 8;      // bf16 elements
    const int stage_u4 = decode_stage_u4(d.dec_nct);              // fragments of a 32-feature tile, then its mu entries
    const size_t n_vdec = (size_t)(p / 32) * stage_u4 * 8;
    std::vector<uint16_t> venc, vdec;
    std::vector<float> negc, mu;
    std::vector<uint32_t> blk(64, 0u), grp(64, 0u);      // whole tables: the kernels fetch all 64 entries
    try {
        venc.assign(n_venc, 0);
        vdec.assign(n_vdec, 0);
        negc.assign((size_t)32 * ntp, 0.0f);
        mu.assign(mu_host, mu_host + p);
    } catch (const std::bad_alloc&) {
        return fail(KVTC_E_NOMEM, "kvtc_plan_create: host allocation failed");
    }
    for (int ks = 0; ks < p / 16; ++ks)
        for (int ct = 0; ct < ntp; ++ct)
            for (int lane = 0; lane < 64; ++lane) {
                const int j = 32 * ct + permuted_index(lane & 31);
                if (j >= r) continue;
                uint16_t* dst = &venc[(((size_t)ks * ntp + ct) * 64 + lane) * 8];
                const int f0 = 16 * ks + 8 * (lane >> 5);
                for (int e = 0; e < 8; ++e) dst[e] = v_kept_host[(size_t)(f0 + e) * ldv + j];
            }
    for (int ft = 0; ft < p / 32; ++ft)
        for (int ks = 0; ks < 2 * d.dec_nct; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                // tiles 2k and 2k+1 hold the even and the odd features of a 64-feature span
                const int f = 64 * (ft >> 1) + 2 * (lane & 31) + (ft & 1);
                const int j0 = 32 * (ks >> 1) + 16 * (lane >> 5) + 8 * (ks & 1);
                uint16_t* dst = &vdec[(((size_t)ft * stage_u4) + (size_t)ks * 64 + lane) * 8];
                for (int e = 0; e < 8; ++e)
                    if (j0 + e < r) dst[e] = v_kept_host[(size_t)f * ldv + j0 + e];
            }
    for (int ft = 0; ft < p / 32; ++ft) {
        float m[32];
        for (int l = 0; l < 32; ++l) m[l] = dec_zero_mu ? 0.0f : mu_host[64 * (ft >> 1) + 2 * l + (ft & 1)];      // the lane order of the tile
        memcpy(&vdec[((size_t)ft * stage_u4 + (size_t)2 * d.dec_nct * 64) * 8], m, sizeof(m));
    }
    for (int j = 0; j < r; ++j) {
        double c = 0.0;
        for (int f = 0; f < p; ++f) c += (double)mu_host[f] * (double)bf16_bits_to_float(v_kept_host[(size_t)f * ldv + j]);
        negc[j] = -(float)c;
    }
    {
        int b = 0;
        long pos = 32L * n_groups;       // bit position of the group's first code
        for (int g = 0; g < n_groups; ++g) {
            const int nb = groups_host[g].n / 16, bits = groups_host[g].bits;
            grp[g] = (uint32_t)b | ((uint32_t)nb << 8) | ((uint32_t)bits << 16);
            for (int k = 0; k < nb; ++k) {
                blk[b + k] = (uint32_t)bits | ((uint32_t)g << 8) | ((uint32_t)(pos / 16) << 16);
                pos += 16L * bits;
            }
            b += nb;
        }
    }

    // ---- one device blob -------------------------------------------------------------
    size_t off = 0;
    const size_t o_desc = off;  off = align_up(off + sizeof(PlanDev), 256);
    const size_t o_venc = off;  off = align_up(off + n_venc * 2, 256);
    const size_t o_vdec = off;  off = align_up(off + n_vdec * 2, 256);
    const size_t o_negc = off;  off = align_up(off + negc.size() * 4, 256);
    const size_t o_mu = off;    off = align_up(off + mu.size() * 4, 256);
    const size_t o_blk = off;   off = align_up(off + blk.size() * 4, 256);
    const size_t o_grp = off;   off = align_up(off + grp.size() * 4, 256);
    char* blob = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&blob), off) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KVTC_E_NOMEM, "kvtc_plan_create: hipMalloc of %zu bytes failed", off);
    }
    d.v_enc = reinterpret_cast<const uint4*>(blob + o_venc);
    d.v_dec = reinterpret_cast<const uint4*>(blob + o_vdec);
    d.negc = reinterpret_cast<const float*>(blob + o_negc);
    d.mu = reinterpret_cast<const float*>(blob + o_mu);
    d.blk = reinterpret_cast<const uint32_t*>(blob + o_blk);
    d.grp = reinterpret_cast<const uint32_t*>(blob + o_grp);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    auto put = [&](size_t o, const void* src, size_t n) {
        if (e == hipSuccess) e = hipMemcpyAsync(blob + o, src, n, hipMemcpyHostToDevice, st);
    };
    put(o_desc, &d, sizeof(d));
    put(o_venc, venc.data(), n_venc * 2);
    put(o_vdec, vdec.data(), n_vdec * 2);
    put(o_negc, negc.data(), negc.size() * 4);
    put(o_mu, mu.data(), mu.size() * 4);
    put(o_blk, blk.data(), blk.size() * 4);
    put(o_grp, grp.data(), grp.size() * 4);
    if (e == hipSuccess) e = hipStreamSynchronize(st);    // the host images die with this call
    if (e != hipSuccess) {
        (void)hipFree(blob);
        return fail(KVTC_E_HIP, "kvtc_plan_create: upload failed: %s", hipGetErrorString(e));
    }
    kvtc_plan* pl = new (std::nothrow) kvtc_plan;
    if (!pl) {
        (void)hipFree(blob);
        return fail(KVTC_E_NOMEM, "kvtc_plan_create: host allocation failed");
    }
    pl->h = d;
    pl->blob = blob;
    pl->desc_dev = reinterpret_cast<PlanDev*>(blob + o_desc);
    pl->record_bytes = (size_t)d.rec_dwords * 4;
    pl->enc_s_wgs = s_wgs;
    pl->enc_s_lds[0] = s_lds[0];
    pl->enc_s_lds[1] = s_lds[1];
    *out = pl;
    return KVTC_OK;
}

void kvtc_plan_destroy(kvtc_plan* plan) {
    if (!plan) return;
    (void)hipFree(plan->blob);
    delete plan;
}

size_t kvtc_record_bytes(const kvtc_plan* plan) { return plan ? plan->record_bytes : 0; }

size_t kvtc_encoded_bytes(const kvtc_plan* plan, int64_t n_tokens) {
    return (plan && n_tokens > 0) ? plan->record_bytes * (size_t)n_tokens : 0;
}

static kvtc_status check_x(const char* who, const void* x, kvtc_dtype dtype, int64_t ld_x, int p) {
    if (!dtype_ok(dtype)) return fail(KVTC_E_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (ld_x < p) return fail(KVTC_E_ARG, "%s: ld_x=%lld < p=%d", who, (long long)ld_x, p);
    if (ld_x > kMaxPitch) return fail(KVTC_E_ARG, "%s: ld_x=%lld above %d", who, (long long)ld_x, kMaxPitch);
    if ((reinterpret_cast<uintptr_t>(x) & 15u) || ((size_t)ld_x * elem_size(dtype)) % 16 != 0)
        return fail(KVTC_E_ARG, "%s: feature array base and row pitch must be 16-byte aligned", who);
    return KVTC_OK;
}

// A feature layout as the kernels take it: token stride, log2 of the block size (0 = contiguous features), and the
// gap between a block's end and the token's next block.
struct XLayout { int64_t ld; int32_t blk_log2; int64_t blk_jump; };

// Checks a kvtc_layout for a tensor of p features (n_tokens < 0: unknown, as in a batched call) and converts it.
static kvtc_status check_layout(const char* who, const void* x, kvtc_dtype dtype, const kvtc_layout* lay, int p, int64_t n_tokens,
                                XLayout* out) {
    if (!lay) return fail(KVTC_E_ARG, "%s: null layout", who);
    if (!dtype_ok(dtype)) return fail(KVTC_E_ARG, "%s: unknown dtype %d", who, (int)dtype);
    const int bf = lay->block_features;
    const int64_t ts = lay->token_stride, bs = lay->block_stride;
    if (bf == 0) {
        kvtc_status st = check_x(who, x, dtype, ts, p);
        if (st != KVTC_OK) return st;
        *out = XLayout{ts, 0, 0};
        return KVTC_OK;
    }
    if (bf < 64 || (bf & (bf - 1)) != 0 || p % bf != 0)
        return fail(KVTC_E_ARG, "%s: block_features=%d must be a power of two, at least 64, that divides p=%d", who, bf, p);
    if (ts < bf || ts > kMaxPitch) return fail(KVTC_E_ARG, "%s: token_stride=%lld outside %d..%d", who, (long long)ts, bf, kMaxPitch);
    if (bs < bf) return fail(KVTC_E_ARG, "%s: block_stride=%lld < block_features=%d", who, (long long)bs, bf);
    const size_t eb = elem_size(dtype);
    if ((reinterpret_cast<uintptr_t>(x) & 15u) || ((size_t)ts * eb) % 16 != 0 || ((size_t)bs * eb) % 16 != 0)
        return fail(KVTC_E_ARG, "%s: feature array base, token stride and block stride must be 16-byte aligned", who);
    // blocks inside a token's row, or tokens inside a block's slab: anything else lets elements overlap
    const int nb = p / bf;
    const bool tokens_major = ts >= (int64_t)(nb - 1) * bs + bf;
    const bool blocks_major = n_tokens < 0 ? bs >= ts : bs >= (n_tokens - 1) * ts + bf;
    if (!tokens_major && !blocks_major)
        return fail(KVTC_E_ARG, "%s: strides (token %lld, block %lld) let elements overlap", who, (long long)ts, (long long)bs);
    int lg = 0;
    while ((1 << lg) < bf) ++lg;
    *out = XLayout{ts, lg, bs - bf};
    return KVTC_OK;
}

static kvtc_status encode_single(const char* who, const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens,
                                 const kvtc_layout* layout, void* out_dev, size_t out_cap, kvtc_stream stream);
static kvtc_status decode_single(const char* who, const kvtc_plan* plan, const void* in_dev, size_t in_bytes, int64_t n_tokens,
                                 void* x_out_dev, kvtc_dtype dtype, const kvtc_layout* layout, kvtc_stream stream, int accumulate = 0,
                                 const float* sum_dev = nullptr, int64_t sum_ld = 0);

kvtc_status kvtc_encode(const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int64_t ld_x,
                        void* out_dev, size_t out_cap, kvtc_stream stream) {
    const kvtc_layout lay = {ld_x, 0, 0, 0};
    return encode_single("kvtc_encode", plan, x_dev, dtype, n_tokens, &lay, out_dev, out_cap, stream);
}
kvtc_status kvtc_encode_blocked(const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens,
                                const kvtc_layout* layout, void* out_dev, size_t out_cap, kvtc_stream stream) {
    return encode_single("kvtc_encode_blocked", plan, x_dev, dtype, n_tokens, layout, out_dev, out_cap, stream);
}
kvtc_status kvtc_decode(const kvtc_plan* plan, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* x_out_dev,
                        kvtc_dtype dtype, int64_t ld_x, kvtc_stream stream) {
    const kvtc_layout lay = {ld_x, 0, 0, 0};
    return decode_single("kvtc_decode", plan, in_dev, in_bytes, n_tokens, x_out_dev, dtype, &lay, stream);
}
kvtc_status kvtc_decode_blocked(const kvtc_plan* plan, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* x_out_dev,
                                kvtc_dtype dtype, const kvtc_layout* layout, kvtc_stream stream) {
    return decode_single("kvtc_decode_blocked", plan, in_dev, in_bytes, n_tokens, x_out_dev, dtype, layout, stream);
}

static kvtc_status encode_single(const char* who, const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens,
                                 const kvtc_layout* layout, void* out_dev, size_t out_cap, kvtc_stream stream) {
    if (!plan) return fail(KVTC_E_ARG, "kvtc_encode: null plan");
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_encode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!x_dev || !out_dev) return fail(KVTC_E_ARG, "kvtc_encode: null buffer");
    XLayout xl;
    kvtc_status st = check_layout(who, x_dev, dtype, layout, plan->h.p, n_tokens, &xl);
    if (st != KVTC_OK) return st;
    if (reinterpret_cast<uintptr_t>(out_dev) & 15u) return fail(KVTC_E_ARG, "kvtc_encode: out_dev must be 16-byte aligned");
    if (out_cap < plan->record_bytes * (size_t)n_tokens)
        return fail(KVTC_E_SMALL, "kvtc_encode: out_cap=%zu < %zu", out_cap, plan->record_bytes * (size_t)n_tokens);
    KernelArgs a;
    memset(&a, 0, sizeof(a));
    a.plans = plan->desc_dev;
    a.n_plans = 1;
    a.jobs = nullptr;
    a.n_jobs = 1;
    a.single = kvtc_job{0, (int32_t)n_tokens, 0};
    a.offsets = nullptr;
    a.x = x_dev;
    a.ld_x = xl.ld;
    a.x_blk_log2 = xl.blk_log2;
    a.x_blk_jump = xl.blk_jump;
    a.stream_buf = out_dev;
    a.cap = out_cap;
    a.status = nullptr;
    // A tensor short enough for all its 64-token tiles to run at once (one wave of workgroups) runs the short-job variant.
    const int64_t tiles_short = (n_tokens + kEncShortTile - 1) / kEncShortTile;
    hipError_t e;
    if (plan->h.enc_s_key != 0 && tiles_short <= (int64_t)cu_count() * plan->enc_s_wgs) {
        a.enc_short = 1;
        a.enc_short_max = 0x7fffffff;
        e = launch_encode(a, dtype, plan->h.enc_s_key, (int)tiles_short, (size_t)kJobTableBytes + 64 + plan->enc_s_lds[dtype], static_cast<hipStream_t>(stream));
    } else {
        const int64_t tiles = (n_tokens + plan->h.enc_tok_wg - 1) / plan->h.enc_tok_wg;
        const int slots = cu_count() * plan->h.enc_wgs;
        const int grid = (int)(tiles < slots ? tiles : slots);
        e = launch_encode(a, dtype, plan->h.enc_nw * 10000 + plan->h.enc_wc * 100 + plan->h.enc_ntw, grid, (size_t)kJobTableBytes + 64 + plan->h.enc_lds[dtype], static_cast<hipStream_t>(stream));
    }
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_encode: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

static kvtc_status decode_single(const char* who, const kvtc_plan* plan, const void* in_dev, size_t in_bytes, int64_t n_tokens,
                                 void* x_out_dev, kvtc_dtype dtype, const kvtc_layout* layout, kvtc_stream stream, int accumulate,
                                 const float* sum_dev, int64_t sum_ld) {
    if (!plan) return fail(KVTC_E_ARG, "kvtc_decode: null plan");
    // accumulate: 0 = store; 1 = add into the fp32 output; 2 = bf16 output = round(sum_dev + product)
    if ((accumulate == 1 && dtype != KVTC_F32) || (accumulate == 2 && (dtype != KVTC_BF16 || !sum_dev || sum_ld < plan->h.p)))
        return fail(KVTC_E_ARG, "%s: bad combination of section mode and output type", who);
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_decode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!in_dev || !x_out_dev) return fail(KVTC_E_ARG, "kvtc_decode: null buffer");
    XLayout xl;
    kvtc_status st = check_layout(who, x_out_dev, dtype, layout, plan->h.p, n_tokens, &xl);
    if (st != KVTC_OK) return st;
    if (reinterpret_cast<uintptr_t>(in_dev) & 15u) return fail(KVTC_E_ARG, "kvtc_decode: in_dev must be 16-byte aligned");
    if (in_bytes < plan->record_bytes * (size_t)n_tokens)
        return fail(KVTC_E_SMALL, "kvtc_decode: in_bytes=%zu < %zu", in_bytes, plan->record_bytes * (size_t)n_tokens);
    KernelArgs a;
    memset(&a, 0, sizeof(a));
    a.plans = plan->desc_dev;
    a.n_plans = 1;
    a.n_jobs = 1;
    a.single = kvtc_job{0, (int32_t)n_tokens, 0};
    a.x = x_out_dev;
    a.ld_x = xl.ld;
    a.x_blk_log2 = xl.blk_log2;
    a.x_blk_jump = xl.blk_jump;
    a.stream_buf = const_cast<void*>(in_dev);
    a.cap = in_bytes;
    a.dec_accumulate = accumulate;
    a.dec_sum = sum_dev;
    a.dec_sum_ld = sum_ld;
    const int slots = cu_count() * plan->h.dec_wgs;
    // A tensor short enough for all its 128-token tiles to run at once takes the variant with one token
    // tile per wave (same plan data: it depends on the padded width only).
    const int64_t tiles_short = (n_tokens + kDecShortTile - 1) / kDecShortTile;
    hipError_t e;
    if (plan->h.dec_tt == 2 && tiles_short <= slots) {
        const DecLayout lay = decode_layout(decode_rec_bytes(1, plan->h.rec_dwords), plan->h.dec_ring_lds, plan->h.dec_wgs);
        a.dec_ring_off = lay.ring_off;
        a.dec_short = 1;
        e = launch_decode(a, dtype, 100 + plan->h.dec_cls, (int)tiles_short, lay.lds_bytes, static_cast<hipStream_t>(stream));
    } else {
        const int64_t tiles = (n_tokens + plan->h.dec_tok_wg - 1) / plan->h.dec_tok_wg;
        const int grid = (int)(tiles < slots ? tiles : slots);
        const DecLayout lay = decode_layout(plan->h.dec_rec_lds, plan->h.dec_ring_lds, plan->h.dec_wgs);
        a.dec_ring_off = lay.ring_off;
        e = launch_decode(a, dtype, plan->h.dec_tt * 100 + plan->h.dec_cls, grid, lay.lds_bytes, static_cast<hipStream_t>(stream));
    }
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_decode: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

kvtc_status kvtc_batch_create(kvtc_batch** out, const kvtc_plan* const* plans, int n_plans, kvtc_stream stream) {
    if (out) *out = nullptr;
    if (!out || !plans || n_plans < 1) return fail(KVTC_E_ARG, "kvtc_batch_create: null argument or no plans");
    std::vector<PlanDev> h;
    kvtc_batch* b = new (std::nothrow) kvtc_batch;
    if (!b) return fail(KVTC_E_NOMEM, "kvtc_batch_create: host allocation failed");
    b->plans_dev = nullptr;
    b->rec_dwords_dev = nullptr;
    b->n_plans = n_plans;
    b->max_p = 0;
    try {
    for (int i = 0; i < n_plans; ++i) {
        if (!plans[i]) {
            delete b;
            return fail(KVTC_E_ARG, "kvtc_batch_create: plan %d is null", i);
        }
        h.push_back(plans[i]->h);
        b->rec_dwords.push_back(plans[i]->h.rec_dwords);
        const PlanDev& ph = plans[i]->h;
        {
            const int key = ph.enc_nw * 10000 + ph.enc_wc * 100 + ph.enc_ntw;
            kvtc_batch::EncVariant* v = nullptr;
            for (auto& e : b->enc)
                if (e.key == key) v = &e;
            if (!v) {
                b->enc.push_back({key, ph.enc_wgs, {0, 0}});
                v = &b->enc.back();
            }
            for (int dt = 0; dt < 2; ++dt)
                if (ph.enc_lds[dt] > v->lds[dt]) v->lds[dt] = ph.enc_lds[dt];
        }
        if (ph.enc_s_key != 0) {
            kvtc_batch::EncVariant* v = nullptr;
            for (auto& e : b->enc_short)
                if (e.key == ph.enc_s_key) v = &e;
            if (!v) {
                b->enc_short.push_back({ph.enc_s_key, plans[i]->enc_s_wgs, {0, 0}});
                v = &b->enc_short.back();
            }
            for (int dt = 0; dt < 2; ++dt)
                if (plans[i]->enc_s_lds[dt] > v->lds[dt]) v->lds[dt] = plans[i]->enc_s_lds[dt];
        }
        {
            const int key = ph.dec_tt * 100 + ph.dec_cls;
            kvtc_batch::DecVariant* v = nullptr;
            for (auto& e : b->dec)
                if (e.key == key) v = &e;
            if (!v) {
                b->dec.push_back({key, ph.dec_wgs, 0, 0});
                v = &b->dec.back();
            }
            if (ph.dec_rec_lds > v->rec) v->rec = ph.dec_rec_lds;
            if (ph.dec_ring_lds > v->ring) v->ring = ph.dec_ring_lds;
        }
        if (ph.p > b->max_p) b->max_p = ph.p;
        {
            bool seen = false;
            for (int v : b->ps) seen = seen || v == ph.p;
            if (!seen) b->ps.push_back(ph.p);
        }
    }
    } catch (const std::bad_alloc&) {
        delete b;
        return fail(KVTC_E_NOMEM, "kvtc_batch_create: host allocation failed");
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&b->plans_dev), sizeof(PlanDev) * n_plans);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&b->rec_dwords_dev), sizeof(uint32_t) * n_plans);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        kvtc_batch_destroy(b);
        return fail(KVTC_E_NOMEM, "kvtc_batch_create: hipMalloc failed");
    }
    e = hipMemcpyAsync(b->plans_dev, h.data(), sizeof(PlanDev) * n_plans, hipMemcpyHostToDevice, st);
    if (e == hipSuccess)
        e = hipMemcpyAsync(b->rec_dwords_dev, b->rec_dwords.data(), sizeof(uint32_t) * n_plans, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        kvtc_batch_destroy(b);
        return fail(KVTC_E_HIP, "kvtc_batch_create: upload failed: %s", hipGetErrorString(e));
    }
    *out = b;
    return KVTC_OK;
}

void kvtc_batch_destroy(kvtc_batch* batch) {
    if (!batch) return;
    if (batch->plans_dev) (void)hipFree(batch->plans_dev);
    if (batch->rec_dwords_dev) (void)hipFree(batch->rec_dwords_dev);
    delete batch;
}

kvtc_status kvtc_offsets(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, uint64_t* offsets_dev,
                         kvtc_stream stream) {
    if (!batch || !offsets_dev || n_jobs < 0 || (n_jobs > 0 && !jobs_dev))
        return fail(KVTC_E_ARG, "kvtc_offsets: null argument or negative job count");
    hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), batch->rec_dwords_dev,
                       batch->n_plans, jobs_dev, n_jobs, offsets_dev, static_cast<uint64_t*>(nullptr));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_offsets: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

kvtc_status kvtc_offsets_append(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, const uint64_t* region_dev,
                                const int64_t* n_coded_dev, uint64_t* offsets_dev, kvtc_stream stream) {
    if (!batch || !offsets_dev || !region_dev || n_jobs < 0 || (n_jobs > 0 && (!jobs_dev || !n_coded_dev)))
        return fail(KVTC_E_ARG, "kvtc_offsets_append: null argument or negative job count");
    hipError_t e = launch_offsets_append(batch->rec_dwords_dev, batch->n_plans, jobs_dev, n_jobs, region_dev, n_coded_dev, offsets_dev,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_offsets_append: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

kvtc_status kvtc_window_split(int64_t ctx, int s, int w, int c, kvtc_split* out) {
    if (!out) return fail(KVTC_E_ARG, "kvtc_window_split: null output");
    if (ctx < 0 || s < 0 || c < 1 || c > w) return fail(KVTC_E_ARG, "kvtc_window_split: need ctx >= 0, s >= 0, 1 <= c <= w (ctx=%lld s=%d w=%d c=%d)", (long long)ctx, s, w, c);
    out->n_sink = ctx < s ? ctx : s;
    const int64_t beyond = ctx - s - (int64_t)(w - c);          // window tokens past the w - c that always stay
    out->n_coded = beyond > 0 ? (beyond / c) * c : 0;
    out->n_window = ctx - out->n_sink - out->n_coded;
    return KVTC_OK;
}

double kvtc_cr_with_window(double ctx, double w, double s, double cr) { return ctx / ((ctx - w - s) / cr + w + s / 2.0); }

kvtc_status kvtc_rope(void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int n_heads, int d_head, int64_t token_stride,
                      int64_t head_stride, const int32_t* positions_dev, int64_t position0, double base, kvtc_rope_pairing pairing,
                      int inverse, kvtc_stream stream) {
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_rope: n_tokens=%lld", (long long)n_tokens);
    if (n_heads < 1 || d_head < 2 || (d_head & 1) || d_head > 256)
        return fail(KVTC_E_ARG, "kvtc_rope: need n_heads >= 1 and an even d_head in 2..256 (n_heads=%d d_head=%d)", n_heads, d_head);
    if (!dtype_ok(dtype)) return fail(KVTC_E_ARG, "kvtc_rope: unknown dtype %d", (int)dtype);
    if (pairing != KVTC_ROPE_HALF && pairing != KVTC_ROPE_INTERLEAVED) return fail(KVTC_E_ARG, "kvtc_rope: unknown pairing %d", (int)pairing);
    if (!(base > 0.0) || !std::isfinite(base)) return fail(KVTC_E_ARG, "kvtc_rope: base must be positive and finite");
    if (inverse != 0 && inverse != 1) return fail(KVTC_E_ARG, "kvtc_rope: inverse must be 0 or 1");
    if (n_tokens == 0) return KVTC_OK;
    if (!x_dev) return fail(KVTC_E_ARG, "kvtc_rope: null buffer");
    // heads and tokens must not overlap: either tokens-major (a token's heads inside its row) or heads-major (a head's tokens inside its slab)
    const bool tokens_major = head_stride >= d_head && token_stride >= (int64_t)(n_heads - 1) * head_stride + d_head;
    const bool heads_major = token_stride >= d_head && head_stride >= (n_tokens - 1) * token_stride + d_head;
    if (!tokens_major && !heads_major)
        return fail(KVTC_E_ARG, "kvtc_rope: strides (token %lld, head %lld) let elements overlap", (long long)token_stride, (long long)head_stride);
    if (reinterpret_cast<uintptr_t>(x_dev) % elem_size(dtype) != 0) return fail(KVTC_E_ARG, "kvtc_rope: misaligned buffer");
    RopeArgs a;
    memset(&a, 0, sizeof(a));
    a.x = x_dev;
    a.n_tokens = n_tokens;
    a.token_stride = token_stride;
    a.head_stride = head_stride;
    a.positions = positions_dev;
    a.position0 = position0;
    a.n_heads = n_heads;
    a.d_head = d_head;
    a.inverse = inverse;
    for (int j = 0; j < d_head / 2; ++j) a.theta[j] = std::pow(base, -2.0 * (double)j / (double)d_head);
    const int64_t items = n_tokens * (int64_t)(d_head / 2);
    const int64_t want = (items + 255) / 256;
    const int64_t cap = (int64_t)cu_count() * 16;
    hipError_t e = launch_rope(a, dtype, pairing == KVTC_ROPE_INTERLEAVED, (int)(want < cap ? want : cap), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_rope: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

kvtc_status kvtc_fp8_pack(const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld_x, void* out_dev, size_t out_cap,
                          kvtc_stream stream) {
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL || p <= 0) return fail(KVTC_E_ARG, "kvtc_fp8_pack: n_tokens=%lld p=%d", (long long)n_tokens, p);
    if (n_tokens == 0) return KVTC_OK;
    if (!x_dev || !out_dev) return fail(KVTC_E_ARG, "kvtc_fp8_pack: null buffer");
    kvtc_status st = check_x("kvtc_fp8_pack", x_dev, dtype, ld_x, p);
    if (st != KVTC_OK) return st;
    if (out_cap < (size_t)n_tokens * (size_t)p) return fail(KVTC_E_SMALL, "kvtc_fp8_pack: out_cap=%zu < %zu", out_cap, (size_t)n_tokens * (size_t)p);
    hipError_t e = launch_fp8_pack(x_dev, dtype, n_tokens, p, ld_x, out_dev, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_fp8_pack: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

kvtc_status kvtc_fp8_unpack(const void* in_dev, size_t in_bytes, int64_t n_tokens, int p, void* x_out_dev, kvtc_dtype dtype,
                            int64_t ld_x, kvtc_stream stream) {
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL || p <= 0) return fail(KVTC_E_ARG, "kvtc_fp8_unpack: n_tokens=%lld p=%d", (long long)n_tokens, p);
    if (n_tokens == 0) return KVTC_OK;
    if (!in_dev || !x_out_dev) return fail(KVTC_E_ARG, "kvtc_fp8_unpack: null buffer");
    kvtc_status st = check_x("kvtc_fp8_unpack", x_out_dev, dtype, ld_x, p);
    if (st != KVTC_OK) return st;
    if (in_bytes < (size_t)n_tokens * (size_t)p) return fail(KVTC_E_SMALL, "kvtc_fp8_unpack: in_bytes=%zu < %zu", in_bytes, (size_t)n_tokens * (size_t)p);
    hipError_t e = launch_fp8_unpack(in_dev, n_tokens, p, x_out_dev, dtype, ld_x, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_fp8_unpack: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

static kvtc_status batch_common(const char* who, const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                                const void* x, kvtc_dtype dtype, const kvtc_layout* layout, const uint64_t* offsets_dev,
                                const void* stream_buf, const uint32_t* status_dev, bool* nothing, XLayout* xl) {
    *nothing = false;
    if (!batch) return fail(KVTC_E_ARG, "%s: null batch", who);
    if (n_jobs < 0) return fail(KVTC_E_ARG, "%s: n_jobs=%d", who, n_jobs);
    if (n_jobs == 0) { *nothing = true; return KVTC_OK; }
    if (n_jobs > kMaxJobs) return fail(KVTC_E_UNSUPPORTED, "%s: %d jobs, at most %d per call", who, n_jobs, kMaxJobs);
    if (!jobs_dev || !x || !offsets_dev || !stream_buf || !status_dev) return fail(KVTC_E_ARG, "%s: null buffer", who);
    if (!layout) return fail(KVTC_E_ARG, "%s: null layout", who);
    for (int pv : batch->ps) {                         // the layout must suit every plan of the batch
        kvtc_status st = check_layout(who, x, dtype, layout, pv, -1, xl);
        if (st != KVTC_OK) return st;
    }
    if (reinterpret_cast<uintptr_t>(stream_buf) & 15u) return fail(KVTC_E_ARG, "%s: stream buffer must be 16-byte aligned", who);
    return KVTC_OK;
}

kvtc_status kvtc_encode_batch(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, const void* x_base_dev,
                              kvtc_dtype dtype, int64_t ld_x, const uint64_t* offsets_dev, void* out_base_dev,
                              size_t out_cap, uint32_t* status_dev, kvtc_stream stream) {
    const kvtc_layout lay = {ld_x, 0, 0, 0};
    return kvtc_encode_batch_blocked(batch, jobs_dev, n_jobs, x_base_dev, dtype, &lay, offsets_dev, out_base_dev, out_cap, status_dev, stream);
}

kvtc_status kvtc_encode_batch_blocked(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, const void* x_base_dev,
                                      kvtc_dtype dtype, const kvtc_layout* layout, const uint64_t* offsets_dev, void* out_base_dev,
                                      size_t out_cap, uint32_t* status_dev, kvtc_stream stream) {
    bool nothing;
    XLayout xl = {0, 0, 0};
    kvtc_status st = batch_common("kvtc_encode_batch", batch, jobs_dev, n_jobs, x_base_dev, dtype, layout, offsets_dev,
                                  out_base_dev, status_dev, &nothing, &xl);
    if (st != KVTC_OK || nothing) return st;
    const int64_t ld_x = xl.ld;
    KernelArgs a;
    memset(&a, 0, sizeof(a));
    a.plans = batch->plans_dev;
    a.n_plans = batch->n_plans;
    a.jobs = jobs_dev;
    a.n_jobs = n_jobs;
    a.offsets = offsets_dev;
    a.x = x_base_dev;
    a.ld_x = ld_x;
    a.x_blk_log2 = xl.blk_log2;
    a.x_blk_jump = xl.blk_jump;
    a.stream_buf = out_base_dev;
    a.cap = out_cap;
    a.status = status_dev;
    // Jobs of at most one 64-token tile go to their plan's short-job variant (one small launch per such
    // variant: a short job is one workgroup), the rest to the bulk variants.
    a.enc_short_max = kEncShortTile;
    a.enc_short = 0;
    for (const auto& v : batch->enc) {
        hipError_t e = launch_encode(a, dtype, v.key, cu_count() * v.wgs,
                                     (size_t)kJobTableBytes + 64 + v.lds[dtype], static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_encode_batch: launch failed: %s", hipGetErrorString(e));
    }
    a.enc_short = 1;
    for (const auto& v : batch->enc_short) {
        const int slots = cu_count() * v.wgs;
        hipError_t e = launch_encode(a, dtype, v.key, n_jobs < slots ? n_jobs : slots,
                                     (size_t)kJobTableBytes + 64 + v.lds[dtype], static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_encode_batch: launch failed: %s", hipGetErrorString(e));
    }
    return KVTC_OK;
}

kvtc_status kvtc_encode_batch_static(const kvtc_plan* const* plans, int n_plans, const kvtc_job* jobs_dev, int n_jobs,
                                     const void* x_base_dev, kvtc_dtype dtype, int64_t ld_x, void* out_base_dev, size_t out_cap,
                                     uint64_t* offsets_out_dev, uint32_t* status_dev, kvtc_stream stream) {
    const char* who = "kvtc_encode_batch_static";
    if (!plans || n_plans < 1) return fail(KVTC_E_ARG, "%s: null argument or no plans", who);
    if (n_plans > kStaticMaxPlans) return fail(KVTC_E_UNSUPPORTED, "%s: %d plans, at most %d per call", who, n_plans, kStaticMaxPlans);
    if (n_jobs < 0) return fail(KVTC_E_ARG, "%s: n_jobs=%d", who, n_jobs);
    if (n_jobs > kMaxJobs) return fail(KVTC_E_UNSUPPORTED, "%s: %d jobs, at most %d per call", who, n_jobs, kMaxJobs);
    if (n_jobs == 0) return KVTC_OK;
    if (!jobs_dev || !x_base_dev || !out_base_dev || !status_dev) return fail(KVTC_E_ARG, "%s: null buffer", who);
    if (!dtype_ok(dtype)) return fail(KVTC_E_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if ((reinterpret_cast<uintptr_t>(x_base_dev) & 15u) || ((size_t)ld_x * elem_size(dtype)) % 16 != 0 || ld_x <= 0)
        return fail(KVTC_E_ARG, "%s: feature array base and row pitch must be 16-byte aligned", who);
    if (ld_x > kMaxPitch) return fail(KVTC_E_ARG, "%s: ld_x=%lld above %d", who, (long long)ld_x, kMaxPitch);
    if (reinterpret_cast<uintptr_t>(out_base_dev) & 15u) return fail(KVTC_E_ARG, "%s: stream buffer must be 16-byte aligned", who);
    // the kernel variants among the plans and their LDS needs, on the stack
    struct Variant { int key, wgs, lds; };
    Variant bulk[kStaticMaxPlans], shrt[kStaticMaxPlans];
    int n_bulk = 0, n_shrt = 0;
    PlanPtrs ptrs;
    for (int i = 0; i < n_plans; ++i) {
        if (!plans[i]) return fail(KVTC_E_ARG, "%s: plan %d is null", who, i);
        const PlanDev& ph = plans[i]->h;
        if (ld_x < ph.p) return fail(KVTC_E_ARG, "%s: ld_x=%lld < p=%d", who, (long long)ld_x, ph.p);
        ptrs.p[i] = plans[i]->desc_dev;
        const int key = ph.enc_nw * 10000 + ph.enc_wc * 100 + ph.enc_ntw;
        int k = 0;
        while (k < n_bulk && bulk[k].key != key) ++k;
        if (k == n_bulk) bulk[n_bulk++] = Variant{key, ph.enc_wgs, 0};
        if (ph.enc_lds[dtype] > bulk[k].lds) bulk[k].lds = ph.enc_lds[dtype];
        if (ph.enc_s_key != 0) {
            k = 0;
            while (k < n_shrt && shrt[k].key != ph.enc_s_key) ++k;
            if (k == n_shrt) shrt[n_shrt++] = Variant{ph.enc_s_key, plans[i]->enc_s_wgs, 0};
            if (plans[i]->enc_s_lds[dtype] > shrt[k].lds) shrt[k].lds = plans[i]->enc_s_lds[dtype];
        }
    }
    for (int i = n_plans; i < kStaticMaxPlans; ++i) ptrs.p[i] = nullptr;
    StaticScratch* sc = nullptr;
    hipError_t e = static_scratch(&sc);
    if (e != hipSuccess) return fail(KVTC_E_HIP, "%s: no address for the static work area: %s", who, hipGetErrorString(e));
    hipStream_t st = static_cast<hipStream_t>(stream);
    // every entry the kernels read is written here first, so nothing of an earlier call is seen
    hipLaunchKernelGGL(gather_plans_kernel, dim3(1), dim3(256), 0, st, ptrs, n_plans, sc);
    hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(256), 0, st, sc->rec_dwords, n_plans, jobs_dev, n_jobs, sc->offsets, offsets_out_dev);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(KVTC_E_HIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    KernelArgs a;
    memset(&a, 0, sizeof(a));
    a.plans = sc->plans;
    a.n_plans = n_plans;
    a.jobs = jobs_dev;
    a.n_jobs = n_jobs;
    a.offsets = sc->offsets;
    a.x = x_base_dev;
    a.ld_x = ld_x;
    a.stream_buf = out_base_dev;
    a.cap = out_cap;
    a.status = status_dev;
    a.enc_short_max = kEncShortTile;
    a.enc_short = 0;
    for (int k = 0; k < n_bulk; ++k) {
        e = launch_encode(a, dtype, bulk[k].key, cu_count() * bulk[k].wgs, (size_t)kJobTableBytes + 64 + bulk[k].lds, st);
        if (e != hipSuccess) return fail(KVTC_E_HIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    }
    a.enc_short = 1;
    for (int k = 0; k < n_shrt; ++k) {
        const int slots = cu_count() * shrt[k].wgs;
        e = launch_encode(a, dtype, shrt[k].key, n_jobs < slots ? n_jobs : slots, (size_t)kJobTableBytes + 64 + shrt[k].lds, st);
        if (e != hipSuccess) return fail(KVTC_E_HIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    }
    return KVTC_OK;
}

kvtc_status kvtc_decode_batch(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, const void* in_base_dev,
                              size_t in_bytes, const uint64_t* offsets_dev, void* x_out_base_dev, kvtc_dtype dtype,
                              int64_t ld_x, uint32_t* status_dev, kvtc_stream stream) {
    const kvtc_layout lay = {ld_x, 0, 0, 0};
    return kvtc_decode_batch_blocked(batch, jobs_dev, n_jobs, in_base_dev, in_bytes, offsets_dev, x_out_base_dev, dtype, &lay, status_dev, stream);
}

kvtc_status kvtc_decode_batch_blocked(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs, const void* in_base_dev,
                                      size_t in_bytes, const uint64_t* offsets_dev, void* x_out_base_dev, kvtc_dtype dtype,
                                      const kvtc_layout* layout, uint32_t* status_dev, kvtc_stream stream) {
    bool nothing;
    XLayout xl = {0, 0, 0};
    kvtc_status st = batch_common("kvtc_decode_batch", batch, jobs_dev, n_jobs, x_out_base_dev, dtype, layout, offsets_dev,
                                  in_base_dev, status_dev, &nothing, &xl);
    if (st != KVTC_OK || nothing) return st;
    const int64_t ld_x = xl.ld;
    KernelArgs a;
    memset(&a, 0, sizeof(a));
    a.plans = batch->plans_dev;
    a.n_plans = batch->n_plans;
    a.jobs = jobs_dev;
    a.n_jobs = n_jobs;
    a.offsets = offsets_dev;
    a.x = x_out_base_dev;
    a.ld_x = ld_x;
    a.x_blk_log2 = xl.blk_log2;
    a.x_blk_jump = xl.blk_jump;
    a.stream_buf = const_cast<void*>(in_base_dev);
    a.cap = in_bytes;
    a.status = status_dev;
    for (const auto& v : batch->dec) {
        const DecLayout lay = decode_layout(v.rec, v.ring, v.wgs);
        a.dec_ring_off = lay.ring_off;
        hipError_t e = launch_decode(a, dtype, v.key, cu_count() * v.wgs, lay.lds_bytes, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_decode_batch: launch failed: %s", hipGetErrorString(e));
    }
    return KVTC_OK;
}

}  // extern "C"

// ---- sectioned plans: more kept coordinates than one record holds ---------------------------------
struct kvtc_wide {
    int p, r;
    std::vector<kvtc_plan*> sections;
    size_t record_bytes;            // over all sections
};

namespace {

constexpr int kSectionCoords = 1024, kSectionGroups = 64;

}  // namespace

extern "C" {

kvtc_status kvtc_wide_create(kvtc_wide** out, int p, int r, const float* mu_host, const uint16_t* v_kept_host, int n_groups,
                             const kvtc_group* groups_host, kvtc_stream stream) {
    if (out) *out = nullptr;
    if (!out || !mu_host || !v_kept_host || !groups_host) return fail(KVTC_E_ARG, "kvtc_wide_create: null argument");
    if (p <= 0 || p % 64 != 0) return fail(KVTC_E_ARG, "kvtc_wide_create: p=%d must be a positive multiple of 64", p);
    if (n_groups < 1 || r < 16) return fail(KVTC_E_ARG, "kvtc_wide_create: r=%d, n_groups=%d", r, n_groups);
    long sum = 0;
    for (int g = 0; g < n_groups; ++g) {
        if (groups_host[g].n < 1 || groups_host[g].n > kSectionCoords)
            return fail(KVTC_E_ARG, "kvtc_wide_create: group %d has %d coordinates (1..%d allowed)", g, (int)groups_host[g].n, kSectionCoords);
        sum += groups_host[g].n;
    }
    if (sum != r) return fail(KVTC_E_ARG, "kvtc_wide_create: group sizes sum to %ld, r=%d", sum, r);
    kvtc_wide* w = new (std::nothrow) kvtc_wide;
    if (!w) return fail(KVTC_E_NOMEM, "kvtc_wide_create: host allocation failed");
    w->p = p;
    w->r = r;
    w->record_bytes = 0;
    // consecutive groups -> sections, greedily: a section takes groups while it stays within 1024 coordinates and 64 groups
    int g0 = 0, j0 = 0;
    while (g0 < n_groups) {
        int g1 = g0, n = 0;
        while (g1 < n_groups && g1 - g0 < kSectionGroups && n + groups_host[g1].n <= kSectionCoords) n += groups_host[g1++].n;
        kvtc_plan* sec = nullptr;
        kvtc_status st = plan_create_impl(&sec, p, n, mu_host, v_kept_host + j0, (size_t)r, g1 - g0, groups_host + g0,
                                          /*dec_zero_mu=*/g0 != 0, stream);
        if (st == KVTC_OK) {
            try { w->sections.push_back(sec); } catch (const std::bad_alloc&) { kvtc_plan_destroy(sec); st = fail(KVTC_E_NOMEM, "kvtc_wide_create: host allocation failed"); }
        }
        if (st != KVTC_OK) {
            kvtc_wide_destroy(w);
            return st;
        }
        w->record_bytes += sec->record_bytes;
        g0 = g1;
        j0 += n;
    }
    *out = w;
    return KVTC_OK;
}

void kvtc_wide_destroy(kvtc_wide* w) {
    if (!w) return;
    for (kvtc_plan* s : w->sections) kvtc_plan_destroy(s);
    delete w;
}

int kvtc_wide_sections(const kvtc_wide* w) { return w ? (int)w->sections.size() : 0; }

size_t kvtc_wide_section_record_bytes(const kvtc_wide* w, int section) {
    return (w && section >= 0 && section < (int)w->sections.size()) ? w->sections[section]->record_bytes : 0;
}

size_t kvtc_wide_record_bytes(const kvtc_wide* w) { return w ? w->record_bytes : 0; }

size_t kvtc_wide_encoded_bytes(const kvtc_wide* w, int64_t n_tokens) {
    if (!w || n_tokens <= 0) return 0;
    size_t pos = 0;
    for (const kvtc_plan* s : w->sections) pos = align_up(pos, 16) + s->record_bytes * (size_t)n_tokens;
    return pos;
}

kvtc_status kvtc_wide_encode(const kvtc_wide* w, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, const kvtc_layout* layout,
                             void* out_dev, size_t out_cap, kvtc_stream stream) {
    if (!w) return fail(KVTC_E_ARG, "kvtc_wide_encode: null plan");
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_wide_encode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!out_dev) return fail(KVTC_E_ARG, "kvtc_wide_encode: null buffer");
    if (out_cap < kvtc_wide_encoded_bytes(w, n_tokens))
        return fail(KVTC_E_SMALL, "kvtc_wide_encode: out_cap=%zu < %zu", out_cap, kvtc_wide_encoded_bytes(w, n_tokens));
    size_t pos = 0;
    for (const kvtc_plan* s : w->sections) {          // a launch per section, each over all tokens
        pos = align_up(pos, 16);
        const size_t bytes = s->record_bytes * (size_t)n_tokens;
        kvtc_status st = encode_single("kvtc_wide_encode", s, x_dev, dtype, n_tokens, layout, static_cast<char*>(out_dev) + pos, bytes, stream);
        if (st != KVTC_OK) return st;
        pos += bytes;
    }
    return KVTC_OK;
}

kvtc_status kvtc_wide_decode(const kvtc_wide* w, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* x_out_dev, kvtc_dtype dtype,
                             const kvtc_layout* layout, float* sum_dev, kvtc_stream stream) {
    if (!w) return fail(KVTC_E_ARG, "kvtc_wide_decode: null plan");
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_wide_decode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!in_dev || !x_out_dev) return fail(KVTC_E_ARG, "kvtc_wide_decode: null buffer");
    if (!dtype_ok(dtype)) return fail(KVTC_E_ARG, "kvtc_wide_decode: unknown dtype %d", (int)dtype);
    if (in_bytes < kvtc_wide_encoded_bytes(w, n_tokens))
        return fail(KVTC_E_SMALL, "kvtc_wide_decode: in_bytes=%zu < %zu", in_bytes, kvtc_wide_encoded_bytes(w, n_tokens));
    // the sections' products are summed in fp32: straight in the output when that is fp32; else in the caller's workspace,
    // from which the last section's launch reads the sum of the others, adds its own part and rounds to bf16 once
    XLayout xl;
    kvtc_status st = check_layout("kvtc_wide_decode", x_out_dev, dtype, layout, w->p, n_tokens, &xl);
    if (st != KVTC_OK) return st;
    const kvtc_layout flat = {w->p, 0, 0, 0};
    const size_t n_sec = w->sections.size();
    if (dtype == KVTC_BF16 && n_sec > 1) {
        if (!sum_dev) return fail(KVTC_E_ARG, "kvtc_wide_decode: bf16 output needs the fp32 workspace sum_dev [n_tokens][p]");
        if (reinterpret_cast<uintptr_t>(sum_dev) & 15u) return fail(KVTC_E_ARG, "kvtc_wide_decode: sum_dev must be 16-byte aligned");
    }
    size_t pos = 0;
    for (size_t c = 0; c < n_sec; ++c) {
        const kvtc_plan* s = w->sections[c];
        pos = align_up(pos, 16);
        const size_t bytes = s->record_bytes * (size_t)n_tokens;
        const char* in = static_cast<const char*>(in_dev) + pos;
        if (dtype == KVTC_F32)
            st = decode_single("kvtc_wide_decode", s, in, bytes, n_tokens, x_out_dev, KVTC_F32, layout, stream, c == 0 ? 0 : 1);
        else if (c + 1 == n_sec)
            st = n_sec == 1 ? decode_single("kvtc_wide_decode", s, in, bytes, n_tokens, x_out_dev, KVTC_BF16, layout, stream)
                            : decode_single("kvtc_wide_decode", s, in, bytes, n_tokens, x_out_dev, KVTC_BF16, layout, stream, 2, sum_dev, w->p);
        else
            st = decode_single("kvtc_wide_decode", s, in, bytes, n_tokens, sum_dev, KVTC_F32, &flat, stream, c == 0 ? 0 : 1);
        if (st != KVTC_OK) return st;
        pos += bytes;
    }
    return KVTC_OK;
}

kvtc_status kvtc_calib_moments(const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int p, const kvtc_layout* layout, double* sum_dev,
                               double* gram_dev, kvtc_stream stream) {
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(KVTC_E_ARG, "kvtc_calib_moments: n_tokens=%lld", (long long)n_tokens);
    if (p <= 0 || p % 64 != 0) return fail(KVTC_E_ARG, "kvtc_calib_moments: p=%d must be a positive multiple of 64", p);
    if (!x_dev || !sum_dev || !gram_dev) return fail(KVTC_E_ARG, "kvtc_calib_moments: null buffer");
    if ((reinterpret_cast<uintptr_t>(sum_dev) & 7u) || (reinterpret_cast<uintptr_t>(gram_dev) & 7u))
        return fail(KVTC_E_ARG, "kvtc_calib_moments: outputs must be 8-byte aligned");
    XLayout xl;
    kvtc_status st = check_layout("kvtc_calib_moments", x_dev, dtype, layout, p, n_tokens, &xl);
    if (st != KVTC_OK) return st;
    const hipError_t e = launch_calib_moments(x_dev, dtype, n_tokens, p, xl.ld, xl.blk_log2, xl.blk_jump, sum_dev, gram_dev,
                                              static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(KVTC_E_HIP, "kvtc_calib_moments: launch failed: %s", hipGetErrorString(e));
    return KVTC_OK;
}

}  // extern "C"
