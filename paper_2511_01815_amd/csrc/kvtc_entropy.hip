// Lossless stage over the packed records for gfx950 (declared in include/kvtc.h, "Lossless stage"):
// a static prefix code per byte position of the record.  (Paper, Section "Entropy coding": the
// quantiser's byte array goes through a lossless coder on the GPU; the paper uses a general-purpose
// DEFLATE, this library a byte-wise entropy coder matched to the records' fixed layout.)
//
// Work decomposition: a wavefront owns a chunk of 64 tokens, a lane one token.  The code tables are
// data (256 code lengths per byte position, from calibration); canonical codes and the decoding
// tables are derived from them on the host at creation.
//   encode = three launches: (1) every lane sums the code lengths of its record's bytes -> len_bits[]
//   and the chunk sizes, written into the container's own directory; (2) one workgroup turns the sizes
//   into offsets; (3) every lane writes its code string into the chunk's image in LDS at the bit
//   offset the lengths before it give (whole dwords OR-ed in), and the wave copies the image out.
//   decode = one launch: the chunk's bit string is staged in LDS, every lane walks its own string with
//   a 12-bit lookup per symbol (tables stay in L2), rows are gathered in LDS and copied out whole.
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
    int record_bytes;
    void* blob;                 // device: enc[R][256] u16, then dec[R][4096] u16
    const uint16_t* enc_dev;    // reversed code | length << 12
    const uint16_t* dec_dev;    // symbol | length << 8, indexed by the next 12 bits of the string
};

namespace {

constexpr int kMaxLen = 12;
constexpr int kChunk = 64;
constexpr int kMaxRecord = 576;       // bytes: a wave's images (chunk string + rows) must fit the LDS

__host__ __device__ inline uint32_t chunk_image_dwords(int R) { return (uint32_t)(kChunk * R * kMaxLen + 31) / 32u; }   // worst case
__host__ __device__ inline uint32_t row_stride_dwords(int R) { return (uint32_t)R / 4u + 1u; }

inline int waves_per_wg(int R) {
    const size_t per_wave = (size_t)chunk_image_dwords(R) * 4 + (size_t)kChunk * row_stride_dwords(R) * 4;
    size_t n = (150u * 1024u) / per_wave;
    return n < 1 ? 1 : (n > 4 ? 4 : (int)n);
}
inline size_t lds_bytes(int R, int waves) {
    return (size_t)waves * ((size_t)chunk_image_dwords(R) * 4 + (size_t)kChunk * row_stride_dwords(R) * 4);
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

// (1) bits of every token's code string -> len_bits[]; bytes of every chunk's bit string -> chunk_off[chunk] (sizes for now)
__global__ void __launch_bounds__(256) entropy_size_kernel(const uint32_t* records, int64_t n_tokens, int R, const uint16_t* enc,
                                                          uint32_t* chunk_off, uint16_t* len_bits, int64_t n_chunks) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t chunk = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    if (chunk >= n_chunks) return;
    const int64_t t = chunk * kChunk + lane;
    uint32_t bits = 0;
    if (t < n_tokens) {
        const uint32_t* row = records + t * (R / 4);
        for (int d = 0; d < R / 4; ++d) {
            const uint32_t w = row[d];
            const uint16_t* e = enc + (size_t)(4 * d) * 256;
            bits += (uint32_t)(e[w & 0xffu] >> 12) + (uint32_t)(e[256 + ((w >> 8) & 0xffu)] >> 12) +
                    (uint32_t)(e[512 + ((w >> 16) & 0xffu)] >> 12) + (uint32_t)(e[768 + (w >> 24)] >> 12);
        }
    }
    len_bits[t] = (uint16_t)bits;                          // the directory has 64 entries per chunk: zero beyond the last token
    const uint32_t total = wave_sum(bits);
    if (lane == 0) chunk_off[chunk] = (total + 31u) / 32u * 4u;
}

// (2) sizes -> offsets, in place; the container's total length -> *out_bytes
__global__ void __launch_bounds__(256) entropy_scan_kernel(uint32_t* chunk_off, int64_t n_chunks, uint64_t header_bytes, uint64_t* out_bytes) {
    __shared__ uint32_t s[256];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < n_chunks; base += 256) {
        const int64_t j = base + tid;
        const uint32_t v = j < n_chunks ? chunk_off[j] : 0u;
        s[tid] = v;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const uint32_t o = tid >= d ? s[tid - d] : 0u;
            __syncthreads();
            s[tid] += o;
            __syncthreads();
        }
        const uint32_t c = carry;
        if (j < n_chunks) chunk_off[j] = c + s[tid] - v;
        __syncthreads();
        if (tid == 255) carry = c + s[255];
        __syncthreads();
    }
    if (tid == 0) {
        chunk_off[n_chunks] = carry;
        if (out_bytes) *out_bytes = header_bytes + carry;
    }
}

// (3) the code strings.  A chunk whose string would end beyond the buffer is left unwritten (the caller sees the
// needed size in *out_bytes).
__global__ void __launch_bounds__(256) entropy_write_kernel(const uint32_t* records, int64_t n_tokens, int R, const uint16_t* enc,
                                                           const uint32_t* chunk_off, const uint16_t* len_bits, int64_t n_chunks,
                                                           uint8_t* payload, uint64_t payload_cap) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t chunk = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    const bool live = chunk < n_chunks;
    const uint32_t img_dw = chunk_image_dwords(R);
    uint32_t* img = lds + (size_t)wave * (img_dw + kChunk * row_stride_dwords(R));
    uint32_t begin = 0, end = 0;
    if (live) { begin = chunk_off[chunk]; end = chunk_off[chunk + 1]; }
    const bool fits = live && end >= begin && (uint64_t)end <= payload_cap && (end - begin) / 4u <= img_dw;
    const uint32_t n_dw = fits ? (end - begin) / 4u : 0u;
    for (uint32_t i = lane; i < n_dw; i += 64) img[i] = 0u;
    __syncthreads();
    if (fits) {
        const int64_t t = chunk * kChunk + lane;
        const uint32_t my_bits = len_bits[t];
        uint32_t pos = wave_exclusive_scan(my_bits);           // bit offset of this token's string in the chunk
        if (t < n_tokens) {
            const uint32_t* row = records + t * (R / 4);
            // the string is built pre-shifted by pos % 32, so that whole dwords of the image are OR-ed in
            uint64_t acc = 0;
            uint32_t nacc = pos & 31u;
            uint32_t dw = pos >> 5;
            for (int d = 0; d < R / 4; ++d) {
                const uint32_t w = row[d];
                const uint16_t* e = enc + (size_t)(4 * d) * 256;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t ent = e[b * 256 + ((w >> (8 * b)) & 0xffu)];
                    acc |= (uint64_t)(ent & 0xfffu) << nacc;
                    nacc += ent >> 12;
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
        uint32_t* out = reinterpret_cast<uint32_t*>(payload + begin);
        for (uint32_t i = lane; i < n_dw; i += 64) out[i] = img[i];
    }
}

// decode: one wave per chunk.  Every read of the input is clamped to the buffer and to the chunk's image, so a
// damaged container gives wrong bytes, never a fault.
__global__ void __launch_bounds__(256) entropy_decode_kernel(const uint32_t* chunk_off, const uint16_t* len_bits, const uint8_t* payload,
                                                            uint64_t payload_cap, int64_t n_tokens, int R, const uint16_t* dec,
                                                            uint32_t* records_out, int64_t n_chunks) {
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t chunk = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;
    const bool live = chunk < n_chunks;
    const uint32_t img_dw = chunk_image_dwords(R), rs = row_stride_dwords(R);
    uint32_t* img = lds + (size_t)wave * (img_dw + kChunk * rs);
    uint32_t* rows = img + img_dw;
    uint32_t n_dw = 0;
    if (live) {
        uint64_t begin = chunk_off[chunk], end = chunk_off[chunk + 1];
        begin = begin < payload_cap ? begin : payload_cap;
        end = end < begin ? begin : (end < payload_cap ? end : payload_cap);
        n_dw = (uint32_t)((end - begin) / 4u);
        n_dw = n_dw < img_dw ? n_dw : img_dw;
        const uint32_t* src = reinterpret_cast<const uint32_t*>(payload + (begin & ~3ull));
        for (uint32_t i = lane; i < n_dw; i += 64) img[i] = src[i];
    }
    __syncthreads();
    if (live) {
        const int64_t t = chunk * kChunk + lane;
        uint32_t pos = wave_exclusive_scan((uint32_t)len_bits[t]);
        if (t < n_tokens) {
            uint32_t* my = rows + (uint32_t)lane * rs;
            for (int d = 0; d < R / 4; ++d) {
                uint32_t w = 0;
                const uint16_t* tab = dec + (size_t)(4 * d) * 4096;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t i0 = pos >> 5, s = pos & 31u;
                    const uint32_t lo = i0 < n_dw ? img[i0] : 0u, hi = i0 + 1u < n_dw ? img[i0 + 1u] : 0u;
                    const uint32_t peek = (uint32_t)((((uint64_t)hi << 32) | lo) >> s) & 0xfffu;
                    const uint32_t ent = tab[b * 4096 + peek];
                    w |= (ent & 0xffu) << (8 * b);
                    pos += ent >> 8;
                }
                my[d] = w;
            }
        }
    }
    __syncthreads();
    if (live) {
        // the chunk's records are contiguous in the output: whole dwords, row by row
        const int64_t t0 = chunk * kChunk;
        const uint32_t n_rows = (uint32_t)((n_tokens - t0) < kChunk ? (n_tokens - t0) : kChunk);
        const uint32_t per_row = (uint32_t)R / 4u;
        uint32_t* out = records_out + t0 * per_row;
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

uint64_t header_bytes(int64_t n_chunks) { return 4ull * (uint64_t)(n_chunks + 1) + 2ull * kChunk * (uint64_t)n_chunks; }

}  // namespace

extern "C" {

kvtc_status kvtc_entropy_create(kvtc_entropy** out, int record_bytes, const uint8_t* code_len_host, kvtc_stream stream) {
    if (out) *out = nullptr;
    if (!out || !code_len_host) return set_error(KVTC_E_ARG, "kvtc_entropy_create: null argument");
    const int R = record_bytes;
    if (R < 4 || R % 4 != 0) return set_error(KVTC_E_ARG, "kvtc_entropy_create: record_bytes=%d must be a positive multiple of 4", R);
    if (R > kMaxRecord) return set_error(KVTC_E_UNSUPPORTED, "kvtc_entropy_create: record_bytes=%d above %d", R, kMaxRecord);
    std::vector<uint16_t> enc, dec;
    try {
        enc.assign((size_t)R * 256, 0);
        dec.assign((size_t)R * 4096, (uint16_t)(1u << 8));          // unused patterns (an incomplete code): symbol 0, one bit
    } catch (const std::bad_alloc&) {
        return set_error(KVTC_E_NOMEM, "kvtc_entropy_create: host allocation failed");
    }
    for (int k = 0; k < R; ++k) {
        const uint8_t* L = code_len_host + (size_t)k * 256;
        // canonical codes: by length, then by symbol (RFC 1951, section 3.2.2); Kraft's inequality must hold
        uint64_t kraft = 0;
        for (int s = 0; s < 256; ++s) {
            if (L[s] < 1 || L[s] > kMaxLen) return set_error(KVTC_E_ARG, "kvtc_entropy_create: position %d, symbol %d: length %d outside 1..%d", k, s, (int)L[s], kMaxLen);
            kraft += 1ull << (kMaxLen - L[s]);
        }
        if (kraft > (1ull << kMaxLen)) return set_error(KVTC_E_ARG, "kvtc_entropy_create: position %d: the lengths are not those of a prefix code", k);
        uint32_t code = 0;
        for (int len = 1; len <= kMaxLen; ++len) {
            for (int s = 0; s < 256; ++s)
                if (L[s] == len) {
                    const uint32_t rev = reverse_bits(code, len);
                    enc[(size_t)k * 256 + s] = (uint16_t)(rev | ((uint32_t)len << 12));
                    for (uint32_t hi = 0; hi < (1u << (kMaxLen - len)); ++hi)
                        dec[(size_t)k * 4096 + (rev | (hi << len))] = (uint16_t)((uint32_t)s | ((uint32_t)len << 8));
                    ++code;
                }
            code <<= 1;
        }
    }
    const size_t enc_b = enc.size() * 2, dec_b = dec.size() * 2;
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
    h->blob = blob;
    h->enc_dev = reinterpret_cast<const uint16_t*>(blob);
    h->dec_dev = reinterpret_cast<const uint16_t*>(blob + enc_b);
    *out = h;
    return KVTC_OK;
}

void kvtc_entropy_destroy(kvtc_entropy* e) {
    if (!e) return;
    (void)hipFree(e->blob);
    delete e;
}

size_t kvtc_entropy_bound(const kvtc_entropy* e, int64_t n_tokens) {
    if (!e || n_tokens <= 0) return 0;
    const int64_t n_chunks = (n_tokens + kChunk - 1) / kChunk;
    return (size_t)header_bytes(n_chunks) + (size_t)n_chunks * chunk_image_dwords(e->record_bytes) * 4;
}

kvtc_status kvtc_entropy_encode(const kvtc_entropy* e, const void* records_dev, int64_t n_tokens, void* out_dev, size_t out_cap,
                                uint64_t* out_bytes_dev, kvtc_stream stream) {
    if (!e) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null tables");
    if (n_tokens < 0) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: n_tokens=%lld", (long long)n_tokens);
    if (!out_bytes_dev) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null out_bytes_dev");
    const int R = e->record_bytes;
    const int64_t n_chunks = (n_tokens + kChunk - 1) / kChunk;
    const uint64_t hdr = header_bytes(n_chunks);
    if (!out_dev || (n_tokens > 0 && !records_dev)) return set_error(KVTC_E_ARG, "kvtc_entropy_encode: null buffer");
    if ((reinterpret_cast<uintptr_t>(records_dev) & 3u) || (reinterpret_cast<uintptr_t>(out_dev) & 3u) || (reinterpret_cast<uintptr_t>(out_bytes_dev) & 7u))
        return set_error(KVTC_E_ARG, "kvtc_entropy_encode: records and output must be 4-byte aligned, out_bytes_dev 8-byte aligned");
    if ((uint64_t)kvtc_entropy_bound(e, n_tokens) - hdr >= (1ull << 32))
        return set_error(KVTC_E_UNSUPPORTED, "kvtc_entropy_encode: %lld tokens of %d bytes may exceed the 4 GiB a container addresses", (long long)n_tokens, R);
    if (out_cap < hdr + 4) return set_error(KVTC_E_SMALL, "kvtc_entropy_encode: out_cap=%zu cannot hold the directory of %llu bytes", out_cap, (unsigned long long)hdr);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t* chunk_off = static_cast<uint32_t*>(out_dev);
    uint16_t* len_bits = reinterpret_cast<uint16_t*>(chunk_off + n_chunks + 1);
    uint8_t* payload = static_cast<uint8_t*>(out_dev) + hdr;
    const int waves = waves_per_wg(R);
    const int grid = (int)((n_chunks + waves - 1) / waves);
    if (n_chunks > 0)
        hipLaunchKernelGGL(entropy_size_kernel, dim3((unsigned)((n_chunks + 3) / 4)), dim3(256), 0, st, static_cast<const uint32_t*>(records_dev),
                           n_tokens, R, e->enc_dev, chunk_off, len_bits, n_chunks);
    hipLaunchKernelGGL(entropy_scan_kernel, dim3(1), dim3(256), 0, st, chunk_off, n_chunks, hdr, out_bytes_dev);
    if (n_chunks > 0) {
        if (allow_full_lds(reinterpret_cast<const void*>(&entropy_write_kernel)) != hipSuccess)
            return set_error(KVTC_E_HIP, "kvtc_entropy_encode: cannot size the LDS");
        hipLaunchKernelGGL(entropy_write_kernel, dim3((unsigned)grid), dim3(64 * waves), lds_bytes(R, waves), st,
                           static_cast<const uint32_t*>(records_dev), n_tokens, R, e->enc_dev, chunk_off, len_bits, n_chunks, payload,
                           (uint64_t)(out_cap - hdr));
    }
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return set_error(KVTC_E_HIP, "kvtc_entropy_encode: launch failed: %s", hipGetErrorString(err));
    return KVTC_OK;
}

kvtc_status kvtc_entropy_decode(const kvtc_entropy* e, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* records_out_dev,
                                size_t out_cap, kvtc_stream stream) {
    if (!e) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: null tables");
    if (n_tokens < 0) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: n_tokens=%lld", (long long)n_tokens);
    if (n_tokens == 0) return KVTC_OK;
    if (!in_dev || !records_out_dev) return set_error(KVTC_E_ARG, "kvtc_entropy_decode: null buffer");
    if ((reinterpret_cast<uintptr_t>(in_dev) & 3u) || (reinterpret_cast<uintptr_t>(records_out_dev) & 3u))
        return set_error(KVTC_E_ARG, "kvtc_entropy_decode: buffers must be 4-byte aligned");
    const int R = e->record_bytes;
    const int64_t n_chunks = (n_tokens + kChunk - 1) / kChunk;
    const uint64_t hdr = header_bytes(n_chunks);
    if (in_bytes < hdr) return set_error(KVTC_E_SMALL, "kvtc_entropy_decode: in_bytes=%zu below the directory's %llu", in_bytes, (unsigned long long)hdr);
    if (out_cap < (size_t)n_tokens * R) return set_error(KVTC_E_SMALL, "kvtc_entropy_decode: out_cap=%zu < %zu", out_cap, (size_t)n_tokens * R);
    const uint32_t* chunk_off = static_cast<const uint32_t*>(in_dev);
    const uint16_t* len_bits = reinterpret_cast<const uint16_t*>(chunk_off + n_chunks + 1);
    const uint8_t* payload = static_cast<const uint8_t*>(in_dev) + hdr;
    const int waves = waves_per_wg(R);
    const int grid = (int)((n_chunks + waves - 1) / waves);
    if (allow_full_lds(reinterpret_cast<const void*>(&entropy_decode_kernel)) != hipSuccess)
        return set_error(KVTC_E_HIP, "kvtc_entropy_decode: cannot size the LDS");
    hipLaunchKernelGGL(entropy_decode_kernel, dim3((unsigned)grid), dim3(64 * waves), lds_bytes(R, waves), static_cast<hipStream_t>(stream),
                       chunk_off, len_bits, payload, (uint64_t)(in_bytes - hdr), n_tokens, R, e->dec_dev, static_cast<uint32_t*>(records_out_dev), n_chunks);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return set_error(KVTC_E_HIP, "kvtc_entropy_decode: launch failed: %s", hipGetErrorString(err));
    return KVTC_OK;
}

}  // extern "C"
