// Lossless stage over the packed records for gfx950 (declared in include/kvtc.h, "Lossless stage"):
// a static prefix code per byte position of the record.  (Paper, Section "Entropy coding": the
// quantiser's byte array goes through a lossless coder on the GPU; the paper uses a general-purpose
// DEFLATE, this library a byte-wise entropy coder matched to the records' fixed layout.)
//
// Work decomposition: a wavefront owns a chunk of 64 tokens, a lane one token; blockIdx.y is the job
// (tensor) of a batched call.  The code tables are data (256 code lengths per byte position and table
// set, from calibration); canonical codes and the decoding tables are derived from them on the host at
// creation.
//   encode = three launches: (1) every lane sums the code lengths of its record's bytes -> len_bits[]
//   and the chunk sizes, written into the container's own directory; (2) a workgroup per job turns the
//   sizes into offsets; (3) every lane writes its code string into the chunk's image in LDS at the bit
//   offset the lengths before it give (whole dwords OR-ed in), and the wave copies the image out.
//   decode = one launch: the chunk's bit string is staged in LDS and every lane walks its own string.
//   The walk depends on nothing but arithmetic: with canonical codes the next 12 bits, read as a
//   number with the first bit on top, are below limit[L] exactly when the code has at most L bits
//   (limit[] = 12 wave-uniform numbers per byte position), so a symbol's length is a count of
//   comparisons, and its rank among the position's symbols follows from one more table entry; the
//   ranks are turned into byte values afterwards, by gathers that wait for nothing.  Rows are
//   collected in LDS and copied out whole.
// Nothing is allocated: the directory lives in the output buffer.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "kvtc_dev.h"

namespace kvtc {
kvtc_status set_error(kvtc_status st, const char* fmt, ...);
}
using namespace kvtc;

struct kvtc_entropy {
    int record_bytes, n_tables;
    void* blob;                 // device: enc[n_tables][R][256] u16, then dec[n_tables][R] DecPos
    const uint16_t* enc_dev;    // reversed code | length << 12
    const void* dec_dev;        // per byte position: limits, rank offsets, symbols by rank
};

namespace {

constexpr int kMaxLen = 12;
constexpr int kChunk = 64;
constexpr int kMaxRecord = 576;       // bytes: a wave's images (chunk string + rows) must fit the LDS
constexpr int kMaxEntropyJobs = 65535;

__host__ __device__ inline uint32_t chunk_image_dwords(int R) { return (uint32_t)(kChunk * R * kMaxLen + 31) / 32u; }   // worst case
__host__ __device__ inline uint32_t row_stride_dwords(int R) { return (uint32_t)R / 4u + 1u; }
__host__ __device__ inline uint64_t header_bytes(int64_t n_chunks) { return 4ull * (uint64_t)(n_chunks + 1) + 2ull * kChunk * (uint64_t)n_chunks; }

// LDS of a launch.  The kernel that writes the code strings holds, per wave, the chunk's image (worst case) and its rows;
// the decoder its rows and, per workgroup, 64 bytes of tables per byte position.  Waves per workgroup: the count (1..4) that
// lets the most waves share a compute unit's 160 KB -- a wave alone on its SIMD has nothing to hide its latencies behind.
inline size_t lds_bytes(int R, int waves, bool decode) {
    const size_t rows = (size_t)kChunk * row_stride_dwords(R) * 4;
    return decode ? (size_t)waves * rows + (size_t)R * 64 : (size_t)waves * ((size_t)chunk_image_dwords(R) * 4 + rows);
}
inline int waves_per_wg(int R, bool decode) {
    int best = 1;
    size_t best_cu = 0;
    for (int n = 1; n <= 4; ++n) {
        const size_t b = lds_bytes(R, n, decode);
        if (b > 150u * 1024u) break;
        size_t wgs = (size_t)kLdsBudget / b;
        if (wgs * n > 32) wgs = 32 / n;                 // a compute unit holds 32 waves at most
        if (wgs * n > best_cu) { best_cu = wgs * n; best = n; }
    }
    return best;
}

// Decoding data of one byte position.  Codes are canonical: those of L bits are first[L] .. first[L] + count[L] - 1.
//   limit[L-1] = (first[L] + count[L]) << (12 - L): the next 12 bits of the string, first bit on top, are below it exactly
//                when the code has at most L bits (non-decreasing in L; entries 12..15 are never reached)
//   off[L-1]   = first[L] - (number of symbols with shorter codes): rank of the symbol = (those 12 bits >> (12 - L)) - off
//   sym[rank]  = byte value, symbols ordered by (length, value)
struct DecPos {
    uint16_t limit[16];
    int16_t off[16];
    uint8_t sym[256];
};
static_assert(sizeof(DecPos) == 320, "layout");

struct EntropyArgs {
    const kvtc_entropy_job* jobs;     // device, or nullptr -> `single`
    int32_t n_jobs;
    kvtc_entropy_job single;
    const uint8_t* records;           // encode: input, decode: output
    uint64_t records_cap;
    uint8_t* coded;                   // encode: output, decode: input
    uint64_t coded_total;
    uint64_t* coded_bytes;            // encode: [n_jobs] container lengths
    const uint16_t* enc;
    const DecPos* dec;
    int32_t R, n_tables;
    int64_t max_tokens;               // the launch covers this many tokens per job; a longer job is left alone
};

// A job as the kernels see it, or ok = false when anything about it is out of range (then the job is left alone).
struct JobView {
    bool ok;
    int64_t T, n_chunks;
    uint32_t* rec;             // the job's records
    uint32_t* chunk_off;       // the container's directory ...
    uint16_t* len_bits;
    uint8_t* payload;          // ... and payload
    uint64_t payload_cap;
    const uint16_t* enc;
    const DecPos* dec;
};
__device__ __forceinline__ JobView job_view(const EntropyArgs& a, int j) {
    const kvtc_entropy_job jb = a.jobs ? a.jobs[j] : a.single;
    JobView v;
    v.T = jb.n_tokens;
    v.n_chunks = ((int64_t)jb.n_tokens + kChunk - 1) / kChunk;
    const uint64_t hdr = header_bytes(v.n_chunks);
    const uint64_t rec_bytes = (uint64_t)(jb.n_tokens > 0 ? jb.n_tokens : 0) * (uint64_t)a.R;
    v.ok = jb.table >= 0 && jb.table < a.n_tables && jb.n_tokens >= 0 && (int64_t)jb.n_tokens <= a.max_tokens && (jb.records_off & 3ull) == 0 && (jb.coded_off & 3ull) == 0 &&
           jb.records_off <= a.records_cap && rec_bytes <= a.records_cap - jb.records_off &&
           jb.coded_off <= a.coded_total && jb.coded_cap <= a.coded_total - jb.coded_off && hdr <= jb.coded_cap;
    if (!v.ok) return v;
    v.rec = reinterpret_cast<uint32_t*>(const_cast<uint8_t*>(a.records) + jb.records_off);
    v.chunk_off = reinterpret_cast<uint32_t*>(a.coded + jb.coded_off);
    v.len_bits = reinterpret_cast<uint16_t*>(v.chunk_off + v.n_chunks + 1);
    v.payload = a.coded + jb.coded_off + hdr;
    v.payload_cap = jb.coded_cap - hdr;
    v.enc = a.enc + (size_t)jb.table * a.R * 256;
    v.dec = a.dec + (size_t)jb.table * a.R;
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}
// exclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_exclusive_scan(uint32_t v) {
    const int lane = threadIdx.x & 63;
    uint32_t s = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(s, d, 64);
        if (lane >= d) s += o;
    }
    return s - v;
}

// The chunk's records, global -> this wave's rows in LDS: whole dwords, coalesced; row r at rows[r * rs].
__device__ __forceinline__ void stage_rows(const JobView& v, int64_t chunk, int R, uint32_t* rows) {
    const int lane = threadIdx.x & 63;
    const int64_t t0 = chunk * kChunk;
    const uint32_t n_rows = (uint32_t)((v.T - t0) < kChunk ? (v.T - t0) : kChunk);
    const uint32_t per_row = (uint32_t)R / 4u, rs = row_stride_dwords(R);
    const uint32_t* src = v.rec + t0 * per_row;
    for (uint32_t i = lane; i < n_rows * per_row; i += 64) {
        const uint32_t r = i / per_row, c = i - r * per_row;
        rows[r * rs + c] = src[i];
    }
}

// (1) bits of every token's code string -> len_bits[]; bytes of every chunk's bit string -> chunk_off[chunk] (sizes for now)
__global__ void __launch_bounds__(256) entropy_size_kernel(const EntropyArgs a) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int R = a.R;
    const JobView v = job_view(a, blockIdx.y);
    const int64_t chunk = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    const bool live = v.ok && chunk < v.n_chunks;
    uint32_t* rows = lds + (size_t)wave * kChunk * row_stride_dwords(R);
    if (live) stage_rows(v, chunk, R, rows);
    __syncthreads();
    if (!live) return;
    const int64_t t = chunk * kChunk + lane;
    uint32_t bits = 0;
    if (t < v.T) {
        const uint32_t* row = rows + (uint32_t)lane * row_stride_dwords(R);
#pragma unroll 4
        for (int d = 0; d < R / 4; ++d) {
            const uint32_t w = row[d];
            const uint16_t* e = v.enc + (size_t)(4 * d) * 256;
            bits += (uint32_t)(e[w & 0xffu] >> 12) + (uint32_t)(e[256 + ((w >> 8) & 0xffu)] >> 12) +
                    (uint32_t)(e[512 + ((w >> 16) & 0xffu)] >> 12) + (uint32_t)(e[768 + (w >> 24)] >> 12);
        }
    }
    v.len_bits[t] = (uint16_t)bits;                        // the directory has 64 entries per chunk: zero beyond the last token
    const uint32_t total = wave_sum(bits);
    if (lane == 0) v.chunk_off[chunk] = (total + 31u) / 32u * 4u;
}

// (2) sizes -> offsets, in place, one workgroup per job; the container's length -> coded_bytes[job] (all ones for a job
// that was left alone)
__global__ void __launch_bounds__(256) entropy_scan_kernel(const EntropyArgs a) {
    __shared__ uint32_t s[256];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x;
    const JobView v = job_view(a, blockIdx.x);
    if (!v.ok) {
        if (tid == 0 && a.coded_bytes) a.coded_bytes[blockIdx.x] = ~0ull;
        return;
    }
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < v.n_chunks; base += 256) {
        const int64_t j = base + tid;
        const uint32_t x = j < v.n_chunks ? v.chunk_off[j] : 0u;
        s[tid] = x;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const uint32_t o = tid >= d ? s[tid - d] : 0u;
            __syncthreads();
            s[tid] += o;
            __syncthreads();
        }
        const uint32_t c = carry;
        if (j < v.n_chunks) v.chunk_off[j] = c + s[tid] - x;
        __syncthreads();
        if (tid == 255) carry = c + s[255];
        __syncthreads();
    }
    if (tid == 0) {
        v.chunk_off[v.n_chunks] = carry;
        if (a.coded_bytes) a.coded_bytes[blockIdx.x] = header_bytes(v.n_chunks) + carry;
    }
}

// (3) the code strings.  A chunk whose string would end beyond the job's room is left unwritten (the caller sees the
// needed size in coded_bytes).
__global__ void __launch_bounds__(256) entropy_write_kernel(const EntropyArgs a) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int R = a.R;
    const JobView v = job_view(a, blockIdx.y);
    const int64_t chunk = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    const bool live = v.ok && chunk < v.n_chunks;
    const uint32_t img_dw = chunk_image_dwords(R), rs = row_stride_dwords(R);
    uint32_t* img = lds + (size_t)wave * (img_dw + kChunk * rs);
    uint32_t* rows = img + img_dw;
    uint32_t begin = 0, end = 0;
    if (live) { begin = v.chunk_off[chunk]; end = v.chunk_off[chunk + 1]; }
    const bool fits = live && end >= begin && (uint64_t)end <= v.payload_cap && (end - begin) / 4u <= img_dw;
    const uint32_t n_dw = fits ? (end - begin) / 4u : 0u;
    for (uint32_t i = lane; i < n_dw; i += 64) img[i] = 0u;
    if (fits) stage_rows(v, chunk, R, rows);
    __syncthreads();
    if (fits) {
        const int64_t t = chunk * kChunk + lane;
        const uint32_t my_bits = v.len_bits[t];
        uint32_t pos = wave_exclusive_scan(my_bits);           // bit offset of this token's string in the chunk
        if (t < v.T) {
            const uint32_t* row = rows + (uint32_t)lane * rs;
            // the string is built pre-shifted by pos % 32, so that whole dwords of the image are OR-ed in
            uint64_t acc = 0;
            uint32_t nacc = pos & 31u;
            uint32_t dw = pos >> 5;
#pragma unroll 4
            for (int d = 0; d < R / 4; ++d) {
                const uint32_t w = row[d];
                const uint16_t* e = v.enc + (size_t)(4 * d) * 256;
                uint32_t ent[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) ent[b] = e[b * 256 + ((w >> (8 * b)) & 0xffu)];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    acc |= (uint64_t)(ent[b] & 0xfffu) << nacc;
                    nacc += ent[b] >> 12;
                    if (nacc >= 32u) {
                        if (dw < n_dw) atomicOr(&img[dw], (uint32_t)acc);
                        ++dw;
                        acc >>= 32;
                        nacc -= 32u;
                    }
                }
            }
            if (nacc != 0u && dw < n_dw) atomicOr(&img[dw], (uint32_t)acc);
        }
    }
    __syncthreads();
    if (fits) {
        uint32_t* out = reinterpret_cast<uint32_t*>(v.payload + begin);
        for (uint32_t i = lane; i < n_dw; i += 64) out[i] = img[i];
    }
}

// decode: one wave per chunk.  Every read of the container is clamped to the job's bytes, so a damaged container gives
// wrong bytes, never a fault.  A lane reads its own bit string straight from the container, one dword ahead of need: the
// strings of a chunk's tokens follow each other, so the wave's reads fall on a few lines that stay in the L1.  LDS: the waves'
// output rows, then the job's limits and rank offsets of every byte position (64 bytes each; the workgroup's chunks belong to
// one job) -- no image of the chunk, which would halve the waves a compute unit can hold.
__global__ void __launch_bounds__(256) entropy_decode_kernel(const EntropyArgs a) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int R = a.R;
    const JobView v = job_view(a, blockIdx.y);
    const int64_t chunk = (int64_t)blockIdx.x * n_waves + wave;
    const bool live = v.ok && chunk < v.n_chunks;
    const uint32_t rs = row_stride_dwords(R);
    uint32_t* rows = lds + (size_t)wave * kChunk * rs;
    uint32_t* tab = lds + (size_t)n_waves * kChunk * rs;          // [R][16] dwords: limit[16] u16, off[16] i16
    if (v.ok) {
        for (int i = threadIdx.x; i < R * 16; i += blockDim.x)
            tab[i] = reinterpret_cast<const uint32_t*>(v.dec + (i >> 4))[i & 15];
    }
    __syncthreads();
    if (live) {
        uint64_t begin = v.chunk_off[chunk], end = v.chunk_off[chunk + 1];
        begin = begin < v.payload_cap ? begin : v.payload_cap;
        end = end < begin ? begin : (end < v.payload_cap ? end : v.payload_cap);
        const uint32_t n_dw = (uint32_t)((end - begin) / 4u);
        const uint32_t* src = reinterpret_cast<const uint32_t*>(v.payload + (begin & ~3ull));
        const int64_t t = chunk * kChunk + lane;
        const uint32_t pos = wave_exclusive_scan((uint32_t)v.len_bits[t]);
        if (t < v.T) {
            uint32_t* my = rows + (uint32_t)lane * rs;
            auto word = [&](uint32_t i) { return i < n_dw ? src[i] : 0u; };
            // the next bits of the string in a register; the container is read a dword ahead of need
            uint32_t idx = (pos >> 5) + 2u;
            uint64_t buf = (((uint64_t)word(idx - 1u) << 32) | word(idx - 2u)) >> (pos & 31u);
            uint32_t nbuf = 64u - (pos & 31u);
            uint32_t ahead = word(idx);
            // pass A: lengths (the only chain) and ranks
            for (int d = 0; d < R / 4; ++d) {
                // the limits of this dword's four positions: wave-uniform LDS reads, fetched before the chain needs them
                uint4 lim[4][2];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint4* T = reinterpret_cast<const uint4*>(tab + (4 * d + b) * 16);
                    lim[b][0] = T[0];
                    lim[b][1] = T[1];
                }
                uint32_t nn[4], hi[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t top = __builtin_bitreverse32((uint32_t)buf) >> 20;        // 12 bits, first bit on top
                    const uint32_t lw[6] = {lim[b][0].x, lim[b][0].y, lim[b][0].z, lim[b][0].w, lim[b][1].x, lim[b][1].y};
                    uint32_t n = 0;
#pragma unroll
                    for (int q = 0; q < 6; ++q) n += (top >= (lw[q] & 0xffffu) ? 1u : 0u) + (top >= (lw[q] >> 16) ? 1u : 0u);
                    const uint32_t len = n < (uint32_t)kMaxLen ? n + 1u : 1u;     // n = 12: a pattern no code starts with (damaged input)
                    nn[b] = n;
                    hi[b] = top >> (12u - len);
                    buf >>= len;
                    nbuf -= len;
                    if (nbuf <= 32u) {
                        buf |= (uint64_t)ahead << nbuf;
                        nbuf += 32u;
                        ++idx;
                        ahead = word(idx);
                    }
                }
                // ranks: (code bits as a number) - off[length - 1]; per-lane LDS reads that the chain does not wait for
                uint32_t w = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int16_t* off = reinterpret_cast<const int16_t*>(tab + (4 * d + b) * 16 + 8);
                    const uint32_t rank = nn[b] < (uint32_t)kMaxLen ? (hi[b] - (uint32_t)(int32_t)off[nn[b]]) & 0xffu : 0u;
                    w |= rank << (8 * b);
                }
                my[d] = w;
            }
            // pass B: ranks -> byte values
#pragma unroll 4
            for (int d = 0; d < R / 4; ++d) {
                const uint32_t w = my[d];
                const DecPos* P = v.dec + 4 * d;
                my[d] = (uint32_t)P[0].sym[w & 0xffu] | ((uint32_t)P[1].sym[(w >> 8) & 0xffu] << 8) |
                        ((uint32_t)P[2].sym[(w >> 16) & 0xffu] << 16) | ((uint32_t)P[3].sym[w >> 24] << 24);
            }
        }
    }
    __syncthreads();
    if (live) {
        // the chunk's records are contiguous in the output: whole dwords, row by row
        const int64_t t0 = chunk * kChunk;
        const uint32_t n_rows = (uint32_t)((v.T - t0) < kChunk ? (v.T - t0) : kChunk);
        const uint32_t per_row = (uint32_t)R / 4u;
        uint32_t* out = v.rec + t0 * per_row;
        for (uint32_t i = lane; i < n_rows * per_row; i += 64) {
            const uint32_t r = i / per_row, c = i - r * per_row;
            out[i] = rows[r * rs + c];
        }
    }
}

uint32_t reverse_bits(uint32_t v, int n) {
    uint32_t r = 0;
    for (int i = 0; i < n; ++i) { r = (r << 1) | (v & 1u); v >>= 1; }
    return r;
}

size_t bound_of(int R, int64_t n_tokens) {
    const int64_t n_chunks = (n_tokens + kChunk - 1) / kChunk;
    return (size_t)header_bytes(n_chunks) + (size_t)n_chunks * chunk_image_dwords(R) * 4;
}

kvtc_status run_encode(const char* who, const kvtc_entropy* e, const EntropyArgs& a_in, int n_jobs, int64_t max_tokens, hipStream_t st) {
    const int R = e->record_bytes;
    const int64_t max_chunks = (max_tokens + kChunk - 1) / kChunk;
    const int waves = waves_per_wg(R, false);
    EntropyArgs a = a_in;
    a.max_tokens = max_tokens;
    if (max_chunks > 0) {
        if (allow_full_lds(reinterpret_cast<const void*>(&entropy_size_kernel)) != hipSuccess)
            return set_error(KVTC_E_HIP, "%s: cannot size the LDS", who);
        hipLaunchKernelGGL(entropy_size_kernel, dim3((unsigned)((max_chunks + 3) / 4), (unsigned)n_jobs), dim3(256),
                           (size_t)4 * kChunk * row_stride_dwords(R) * 4, st, a);
    }
    hipLaunchKernelGGL(entropy_scan_kernel, dim3((unsigned)n_jobs), dim3(256), 0, st, a);
    if (max_chunks > 0) {
        if (allow_full_lds(reinterpret_cast<const void*>(&entropy_write_kernel)) != hipSuccess)
            return set_error(KVTC_E_HIP, "%s: cannot size the LDS", who);
        hipLaunchKernelGGL(entropy_write_kernel, dim3((unsigned)((max_chunks + waves - 1) / waves), (unsigned)n_jobs), dim3(64 * waves),
                           lds_bytes(R, waves, false), st, a);
    }
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return set_error(KVTC_E_HIP, "%s: launch failed: %s", who, hipGetErrorString(err));
    return KVTC_OK;
}

kvtc_status run_decode(const char* who, const kvtc_entropy* e, const EntropyArgs& a_in, int n_jobs, int64_t max_tokens, hipStream_t st) {
    const int R = e->record_bytes;
    EntropyArgs a = a_in;
    a.max_tokens = max_tokens;
    const int64_t max_chunks = (max_tokens + kChunk - 1) / kChunk;
    if (max_chunks == 0) return KVTC_OK;
    const int waves = waves_per_wg(R, true);
    if (allow_full_lds(reinterpret_cast<const void*>(&entropy_decode_kernel)) != hipSuccess)
        return set_error(KVTC_E_HIP, "%s: cannot size the LDS", who);
    hipLaunchKernelGGL(entropy_decode_kernel, dim3((unsigned)((max_chunks + waves - 1) / waves), (unsigned)n_jobs), dim3(64 * waves),
                       lds_bytes(R, waves, true), st, a);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return set_error(KVTC_E_HIP, "%s: launch failed: %s", who, hipGetErrorString(err));
    return KVTC_OK;
}

EntropyArgs base_args(const kvtc_entropy* e) {
    EntropyArgs a;
    memset(&a, 0, sizeof(a));
    a.enc = e->enc_dev;
    a.dec = static_cast<const DecPos*>(e->dec_dev);
    a.R = e->record_bytes;
    a.n_tables = e->n_tables;
    return a;
}

}  // namespace

extern "C" {

kvtc_status kvtc_entropy_create(kvtc_entropy** out, int record_bytes, int n_tables, const uint8_t* code_len_host, kvtc_stream stream) {
    if (out) *out = nullptr;
    if (!out || !code_len_host) return set_error(KVTC_E_ARG, "kvtc_entropy_create: null argument");
    const int R = record_bytes;
    if (R < 4 || R % 4 != 0) return set_error(KVTC_E_ARG, "kvtc_entropy_create: record_bytes=%d must be a positive multiple of 4", R);
    if (R > kMaxRecord) return set_error(KVTC_E_UNSUPPORTED, "kvtc_entropy_create: record_bytes=%d above %d", R, kMaxRecord);
    if (n_tables < 1 || n_tables > 4096) return set_error(KVTC_E_ARG, "kvtc_entropy_create: n_tables=%d outside 1..4096", n_tables);
    const size_t rows = (size_t)n_tables * R;
    std::vector<uint16_t> enc;
    std::vector<DecPos> dec;
    try {
        enc.assign(rows * 256, 0);
        dec.resize(rows);
    } catch (const std::bad_alloc&) {
        return set_error(KVTC_E_NOMEM, "kvtc_entropy_create: host allocation failed");
    }
    for (size_t k = 0; k < rows; ++k) {
        const uint8_t* L = code_len_host + k * 256;
        // canonical codes: by length, then by symbol (RFC 1951, section 3.2.2); Kraft's inequality must hold
        uint64_t kraft = 0;
        for (int s = 0; s < 256; ++s) {
            if (L[s] < 1 || L[s] > kMaxLen)
                return set_error(KVTC_E_ARG, "kvtc_entropy_create: table %d, position %d, symbol %d: length %d outside 1..%d", (int)(k / R), (int)(k % R), s, (int)L[s], kMaxLen);
            kraft += 1ull << (kMaxLen - L[s]);
        }
        if (kraft > (1ull << kMaxLen))
            return set_error(KVTC_E_ARG, "kvtc_entropy_create: table %d, position %d: the lengths are not those of a prefix code", (int)(k / R), (int)(k % R));
        DecPos& D = dec[k];
        memset(&D, 0, sizeof(D));
        for (int i = kMaxLen; i < 16; ++i) D.limit[i] = 0xffffu;
        uint32_t code = 0, rank = 0;
        for (int len = 1; len <= kMaxLen; ++len) {
            D.off[len - 1] = (int16_t)((int32_t)code - (int32_t)rank);       // first code of this length - symbols with shorter codes
            for (int s = 0; s < 256; ++s)
                if (L[s] == len) {
                    enc[k * 256 + s] = (uint16_t)(reverse_bits(code, len) | ((uint32_t)len << 12));
                    D.sym[rank++] = (uint8_t)s;
                    ++code;
                }
            D.limit[len - 1] = (uint16_t)(code << (kMaxLen - len));           // at most 4096
            code <<= 1;
        }
    }
    const size_t enc_b = enc.size() * 2, dec_b = dec.size() * sizeof(DecPos);
    char* blob = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&blob), enc_b + dec_b) != hipSuccess) {
        (void)hipGetLastError();
        return set_error(KVTC_E_NOMEM, "kvtc_entropy_create: hipMalloc of %zu bytes failed", enc_b + dec_b);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(blob, enc.data(), enc_b, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(blob + enc_b, dec.data(), dec_b, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);           // the host images die with this call
    kvtc_entropy* h = e == hipSuccess ? new (std::nothrow) kvtc_entropy : nullptr;
    if (!h) {
        (void)hipFree(blob);
        return e != hipSuccess ? set_error(KVTC_E_HIP, "kvtc_entropy_create: upload failed: %s", hipGetErrorString(e))
                               : set_error(KVTC_E_NOMEM, "kvtc_entropy_create: host allocation failed");
    }
    h->record_bytes = R;
    h->n_tables = n_tables;
    h->blob = blob;
    h->enc_dev = reinterpret_cast<const uint16_t*>(blob);
    h->dec_dev = blob + enc_b;
    *out = h;
    return KVTC_OK;
}

void kvtc_entropy_destroy(kvtc_entropy* e) {
    if (!e) return;
    (void)hipFree(e->blob);
    delete e;
}

size_t kvtc_entropy_bound(const kvtc_entropy* e, int64_t n_tokens) {
    if (!e || n_tokens <= 0) return e ? (size_t)header_bytes(0) : 0;
    return bound_of(e->record_bytes, n_tokens);
}

kvtc_status kvtc_entropy_encode(const kvtc_entropy* e, int table, const void* records_dev, int64_t n_tokens, void* out_dev, size_t out_cap,
                                uint64_t* out_bytes_dev, kvtc_stream stream) {
    if (!e) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null tables");
    if (table < 0 || table >= e->n_tables) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: table=%d outside 0..%d", table, e->n_tables - 1);
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: n_tokens=%lld", (long long)n_tokens);
    if (!out_bytes_dev) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null out_bytes_dev");
    const int R = e->record_bytes;
    const int64_t n_chunks = (n_tokens + kChunk - 1) / kChunk;
    const uint64_t hdr = header_bytes(n_chunks);
    if (!out_dev || (n_tokens > 0 && !records_dev)) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null buffer");
    if ((reinterpret_cast<uintptr_t>(records_dev) & 3u) || (reinterpret_cast<uintptr_t>(out_dev) & 3u) || (reinterpret_cast<uintptr_t>(out_bytes_dev) & 7u))
        return set_error(KVTC_E_ARG, "kvtc_entropy_encode: records and output must be 4-byte aligned, out_bytes_dev 8-byte aligned");
    if ((uint64_t)bound_of(R, n_tokens) - hdr >= (1ull << 32))
        return set_error(KVTC_E_UNSUPPORTED, "kvtc_entropy_encode: %lld tokens of %d bytes may exceed the 4 GiB a container addresses", (long long)n_tokens, R);
    if (out_cap < hdr) return set_error(KVTC_E_SMALL, "kvtc_entropy_encode: out_cap=%zu cannot hold the directory of %llu bytes", out_cap, (unsigned long long)hdr);
    EntropyArgs a = base_args(e);
    a.n_jobs = 1;
    a.single = kvtc_entropy_job{table, (int32_t)n_tokens, 0, 0, out_cap};
    a.records = static_cast<const uint8_t*>(records_dev);
    a.records_cap = (uint64_t)n_tokens * R;
    a.coded = static_cast<uint8_t*>(out_dev);
    a.coded_total = out_cap;
    a.coded_bytes = out_bytes_dev;
    return run_encode("kvtc_entropy_encode", e, a, 1, n_tokens, static_cast<hipStream_t>(stream));
}

kvtc_status kvtc_entropy_decode(const kvtc_entropy* e, int table, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* records_out_dev,
                                size_t out_cap, kvtc_stream stream) {
    if (!e) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: null tables");
    if (table < 0 || table >= e->n_tables) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: table=%d outside 0..%d", table, e->n_tables - 1);
    if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!in_dev || !records_out_dev) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: null buffer");
    if ((reinterpret_cast<uintptr_t>(in_dev) & 3u) || (reinterpret_cast<uintptr_t>(records_out_dev) & 3u))
        return set_error(KVTC_E_ARG, "kvtc_entropy_decode: buffers must be 4-byte aligned");
    const int R = e->record_bytes;
    const uint64_t hdr = header_bytes((n_tokens + kChunk - 1) / kChunk);
    if (in_bytes < hdr) return set_error(KVTC_E_SMALL, "kvtc_entropy_decode: in_bytes=%zu below the directory's %llu", in_bytes, (unsigned long long)hdr);
    if (out_cap < (size_t)n_tokens * R) return set_error(KVTC_E_SMALL, "kvtc_entropy_decode: out_cap=%zu < %zu", out_cap, (size_t)n_tokens * R);
    EntropyArgs a = base_args(e);
    a.n_jobs = 1;
    a.single = kvtc_entropy_job{table, (int32_t)n_tokens, 0, 0, in_bytes};
    a.records = static_cast<const uint8_t*>(records_out_dev);
    a.records_cap = (uint64_t)n_tokens * R;
    a.coded = static_cast<uint8_t*>(const_cast<void*>(in_dev));
    a.coded_total = in_bytes;
    return run_decode("kvtc_entropy_decode", e, a, 1, n_tokens, static_cast<hipStream_t>(stream));
}

static kvtc_status batch_checks(const char* who, const kvtc_entropy* e, const kvtc_entropy_job* jobs_dev, int n_jobs, int64_t max_tokens,
                                const void* records, const void* coded, bool* nothing) {
    *nothing = false;
    if (!e) return set_error(KVTC_E_ARG, "%s: null tables", who);
    if (n_jobs < 0 || max_tokens < 0 || max_tokens > 0x7fffffffLL) return set_error(KVTC_E_ARG, "%s: n_jobs=%d, max_tokens=%lld", who, n_jobs, (long long)max_tokens);
    if (n_jobs == 0) { *nothing = true; return KVTC_OK; }
    if (n_jobs > kMaxEntropyJobs) return set_error(KVTC_E_UNSUPPORTED, "%s: %d jobs, at most %d per call", who, n_jobs, kMaxEntropyJobs);
    if (!jobs_dev || !records || !coded) return set_error(KVTC_E_ARG, "%s: null buffer", who);
    if ((reinterpret_cast<uintptr_t>(records) & 3u) || (reinterpret_cast<uintptr_t>(coded) & 3u) || (reinterpret_cast<uintptr_t>(jobs_dev) & 7u))
        return set_error(KVTC_E_ARG, "%s: buffers must be 4-byte aligned, the job table 8-byte aligned", who);
    if ((uint64_t)bound_of(e->record_bytes, max_tokens) >= (1ull << 32))
        return set_error(KVTC_E_UNSUPPORTED, "%s: %lld tokens of %d bytes may exceed the 4 GiB a container addresses", who, (long long)max_tokens, e->record_bytes);
    return KVTC_OK;
}

kvtc_status kvtc_entropy_encode_batch(const kvtc_entropy* e, const kvtc_entropy_job* jobs_dev, int n_jobs, int64_t max_tokens,
                                      const void* records_base_dev, size_t records_bytes, void* coded_base_dev, size_t coded_cap,
                                      uint64_t* coded_bytes_dev, kvtc_stream stream) {
    bool nothing;
    kvtc_status st = batch_checks("kvtc_entropy_encode_batch", e, jobs_dev, n_jobs, max_tokens, records_base_dev, coded_base_dev, &nothing);
    if (st != KVTC_OK || nothing) return st;
    if (!coded_bytes_dev || (reinterpret_cast<uintptr_t>(coded_bytes_dev) & 7u))
        return set_error(KVTC_E_ARG, "kvtc_entropy_encode_batch: coded_bytes_dev must be an 8-byte aligned device array");
    EntropyArgs a = base_args(e);
    a.jobs = jobs_dev;
    a.n_jobs = n_jobs;
    a.records = static_cast<const uint8_t*>(records_base_dev);
    a.records_cap = records_bytes;
    a.coded = static_cast<uint8_t*>(coded_base_dev);
    a.coded_total = coded_cap;
    a.coded_bytes = coded_bytes_dev;
    return run_encode("kvtc_entropy_encode_batch", e, a, n_jobs, max_tokens, static_cast<hipStream_t>(stream));
}

kvtc_status kvtc_entropy_decode_batch(const kvtc_entropy* e, const kvtc_entropy_job* jobs_dev, int n_jobs, int64_t max_tokens,
                                      const void* coded_base_dev, size_t coded_bytes, void* records_base_dev, size_t records_cap,
                                      kvtc_stream stream) {
    bool nothing;
    kvtc_status st = batch_checks("kvtc_entropy_decode_batch", e, jobs_dev, n_jobs, max_tokens, records_base_dev, coded_base_dev, &nothing);
    if (st != KVTC_OK || nothing) return st;
    EntropyArgs a = base_args(e);
    a.jobs = jobs_dev;
    a.n_jobs = n_jobs;
    a.records = static_cast<const uint8_t*>(records_base_dev);
    a.records_cap = records_cap;
    a.coded = static_cast<uint8_t*>(const_cast<void*>(coded_base_dev));
    a.coded_total = coded_bytes;
    return run_decode("kvtc_entropy_decode_batch", e, a, n_jobs, max_tokens, static_cast<hipStream_t>(stream));
}

}  // extern "C"
