// libpcc: kernels and C ABI (see include/pcc.h for the contract).
//
// Kernels
//   encode_kernel      gather + network (MFMA) + mixture -> (start,freq) of the
//                      true sub-pixels, all pixels in parallel
//   rans_rows_kernel   one lane per image row: push the row's symbols last to
//                      first into a per-row slab, written backwards
//   scan_kernel        exclusive prefix sum of row payload sizes, header, offsets
//   compact_kernel     slabs -> contiguous stream
//   decode_kernel      persistent wavefront decoder: one workgroup (4 waves) per
//                      band of 16 rows, step t handles pixel (r, t - 2r) of each row
//   cdf_tables_kernel  test hook: full integer CDF tables from given parameters
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "pcc.h"
#include "pcc_device.h"

namespace pcc {

constexpr uint32_t kBlobMagic = 0x57434350u;    // "PCCW"
constexpr uint32_t kStreamMagic = 0x31434350u;  // "PCC1"
constexpr int kStreamHeader = 32;
constexpr uint32_t kModelTag = 5u | (10u << 8) | (2u << 16) | (16u << 24);
constexpr int kBandRows = 16;
constexpr uint32_t kMailTag = 0x80000000u;
// Encode kernel variants: tiles of 16 pixels per wave per iteration x threads per workgroup.
// More tiles per wave reuse each LDS weight read more often but need more registers
// (4 tiles only fit with one wave per SIMD).
struct EncodeVariant { int tiles, threads; };
constexpr EncodeVariant kEncodeVariants[3] = {{1, 512}, {2, 512}, {1, 1024}};
constexpr int kDefaultEncodeVariant = 1;

// status words in device memory
enum { kStErr = 0, kStAbort = 1, kStTicket = 2, kStWords = 4 };

__host__ __device__ inline size_t slab_words(int W) { return (6 * (size_t)W + 16) / 4 + 1; }

// ---------------------------------------------------------------------------
// shared device helpers
// ---------------------------------------------------------------------------

__device__ __forceinline__ void set_error(int* status, int code) { atomicCAS(&status[kStErr], 0, code); }

// An offset of zero the optimiser cannot see through.  Added to the LDS base
// inside a loop it keeps the (loop-invariant) weight reads from being hoisted
// out of the loop and parked in registers or scratch.
__device__ __forceinline__ uint32_t opaque_zero() {
    uint32_t z = 0;
    asm volatile("" : "+s"(z));
    return z;
}

__device__ __forceinline__ void copy_model_to_lds(uint8_t* lds, const uint8_t* __restrict__ model) {
    const uint4* src = reinterpret_cast<const uint4*>(model);
    uint4* dst = reinterpret_cast<uint4*>(lds);
    for (int i = threadIdx.x; i < kModelBytes / 16; i += blockDim.x) dst[i] = src[i];
}

// Source of slot i of lane group g in the first-layer operand: row offset and
// byte within the row's neighbour run (which starts at column c-2).
__device__ __forceinline__ void slot_source(int g, int i, int& dr, int& b, bool& used) {
    if (i < 4) {
        dr = (g < 2) ? -2 : -1;
        b = (g & 1) ? 8 + i : i;
        used = true;
    } else {
        dr = (g & 1) ? 0 : ((g == 0) ? -2 : -1);
        b = (g == 1) ? i - 4 : i;
        used = !(g == 3 && i >= 6);
    }
}

// Raw head registers of one lane after the network -> mixture of "its" channel
// (lane groups 0,1,2 = R,G,B) with the coupling coefficients pulled from group 3.
struct LaneHead {
    ChanParams cp;
    float c1[5];  // alpha (group 1) or beta (group 2)
    float c2[5];  // gamma (group 2)
};

__device__ __forceinline__ void lane_head_setup(const f32x4_t (&o)[kL4_OB], int lane, float lut_scale, LaneHead& h) {
    float v[16];
#pragma unroll
    for (int ob = 0; ob < kL4_OB; ++ob) {
        v[4 * ob + 0] = o[ob].x; v[4 * ob + 1] = o[ob].y; v[4 * ob + 2] = o[ob].z; v[4 * ob + 3] = o[ob].w;
    }
    const int g = lane >> 4;
    const int src = (lane & 15) + 48;
    float x3[13];
#pragma unroll
    for (int s = 0; s < 13; ++s) x3[s] = __shfl(v[s], src);
    float raw[15];
#pragma unroll
    for (int s = 0; s < 15; ++s) raw[s] = v[s];
    channel_setup(raw, lut_scale, h.cp);
    h.c1[0] = v[15];
#pragma unroll
    for (int k = 1; k < 5; ++k) h.c1[k] = (g == 1) ? x3[k - 1] : x3[3 + k];
#pragma unroll
    for (int k = 0; k < 5; ++k) h.c2[k] = x3[8 + k];
}

// ---------------------------------------------------------------------------
// encode: all pixels in parallel
// ---------------------------------------------------------------------------
template <int T, int THREADS>
__global__ void __launch_bounds__(THREADS)
encode_kernel(const uint8_t* __restrict__ model, const uint8_t* __restrict__ img, int H, int W, uint32_t P,
              uint32_t* __restrict__ sf, float* __restrict__ params, float* __restrict__ bits, int* status) {
    extern __shared__ __align__(16) uint8_t lds[];
    copy_model_to_lds(lds, model);
    __syncthreads();
    const float2* lut = reinterpret_cast<const float2*>(lds + kLutOff);
    const float lut_scale = *reinterpret_cast<const float*>(lds + kLutScaleOff);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int g = lane >> 4, nl = lane & 15;
    const uint32_t groups = (P + 16 * T - 1) / (16 * T);

    for (uint32_t grp = blockIdx.x * nwaves + wave; grp < groups; grp += gridDim.x * nwaves) {
        u32x4_t in[T][1][2];
        uint32_t pix[T];   // the pixel's own bytes r | g<<8 | b<<16
        // This lane's eight first-layer inputs are two runs of four consecutive image bytes:
        // (row offset, byte offset within the 12-byte window of columns c-2..c+1).
        const int drA = (g < 2) ? -2 : -1, offA = (g & 1) ? 8 : 0;
        const int drB = (g == 0) ? -2 : (g == 2 ? -1 : 0), offB = (g == 1) ? 0 : 4;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t p = grp * (16 * T) + 16 * t + nl;
            uint32_t runA = 0, runB = 0;
            pix[t] = 0;
            if (p < P) {
                const uint32_t rowg = p / (uint32_t)W;
                const int c = (int)(p - rowg * (uint32_t)W);
                const uint32_t im = rowg / (uint32_t)H;
                const int r = (int)(rowg - im * (uint32_t)H);
                const uint8_t* base = img + (size_t)im * H * W * 3;
                const int me = (r * W + c) * 3;
                if (p + 1 < P) {
                    uint32_t v;
                    __builtin_memcpy(&v, base + me, 4);       // unaligned dword; the fourth byte is the next pixel's
                    pix[t] = v & 0xFFFFFFu;
                } else {
                    pix[t] = (uint32_t)base[me] | ((uint32_t)base[me + 1] << 8) | ((uint32_t)base[me + 2] << 16);
                }
                // a run is read with one load when all its bytes lie in the image, byte by byte at the borders
                auto load_run = [&](int dr, int off) -> uint32_t {
                    const int rr = r + dr;
                    const int col0 = c - 2 + (off >> 2);          // the run touches columns col0 and col0 + 1
                    const int at = (rr * W + (c - 2)) * 3 + off;
                    uint32_t v = 0;
                    if (rr >= 0 && col0 >= 0 && col0 + 1 < W) {
                        __builtin_memcpy(&v, base + at, 4);
                    } else if (rr >= 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int col = c - 2 + (((off + i) * 11) >> 5);
                            if (col >= 0 && col < W) v |= (uint32_t)base[at + i] << (8 * i);
                        }
                    }
                    return v;
                };
                runA = load_run(drA, offA);
                runB = load_run(drB, offB);
            }
            // bytes -> bf16 (exact): the upper halves of the fp32 conversions, packed in pairs
            const uint32_t sel = 0x07060302u;
            in[t][0][0].x = __builtin_amdgcn_perm(__float_as_uint((float)((runA >> 8) & 0xFFu)), __float_as_uint((float)(runA & 0xFFu)), sel);
            in[t][0][0].y = __builtin_amdgcn_perm(__float_as_uint((float)(runA >> 24)), __float_as_uint((float)((runA >> 16) & 0xFFu)), sel);
            in[t][0][0].z = __builtin_amdgcn_perm(__float_as_uint((float)((runB >> 8) & 0xFFu)), __float_as_uint((float)(runB & 0xFFu)), sel);
            in[t][0][0].w = __builtin_amdgcn_perm(__float_as_uint((float)(runB >> 24)), __float_as_uint((float)((runB >> 16) & 0xFFu)), sel);
            in[t][0][1] = in[t][0][0];   // unused (layer-1 inputs are exact)
        }

        f32x4_t out[T][kL4_OB];
        mlp_forward<T, (T == 1 && THREADS <= 512 ? 10 : 2), (T == 1 && THREADS <= 512 ? 8 : 2)>(lds + opaque_zero(), lane, in, out);

#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t p = grp * (16 * T) + 16 * t + nl;
            const bool live = p < P;
            if (params != nullptr && live) {
#pragma unroll
                for (int ob = 0; ob < kL4_OB; ++ob) {
                    const float vv[4] = {out[t][ob].x, out[t][ob].y, out[t][ob].z, out[t][ob].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int idx = head_index(g, 4 * ob + i);
                        if (idx >= 0) params[(size_t)p * PCC_HEAD_OUTPUTS + idx] = vv[i];
                    }
                }
            }
            LaneHead h;
            lane_head_setup(out[t], lane, lut_scale, h);
            const float rhat = (float)(pix[t] & 0xFF) * (1.0f / 256.0f);
            const float ghat = (float)((pix[t] >> 8) & 0xFF) * (1.0f / 256.0f);
            if (g == 1) couple_green(h.cp, h.c1, rhat);
            if (g == 2) couple_blue(h.cp, h.c1, h.c2, rhat, ghat);
            const int x = (int)((pix[t] >> (8 * (g & 3))) & 0xFF);   // group 3 reads the zero top byte
            const uint32_t lo = cq_full(h.cp, x, lut);
            const uint32_t hi = cq_full(h.cp, x + 1, lut);
            uint32_t freq = hi - lo;
            if (g < 3 && live && (hi <= lo || freq > 65536u)) { set_error(status, PCC_E_INTERNAL); freq = 1; }
            if (sf != nullptr && g < 3 && live) sf[(size_t)p * 3 + g] = lo | ((freq - 1u) << 16);
            if (bits != nullptr) {
                const float mine = 16.0f - __builtin_amdgcn_logf((float)freq);
                const float tot = (__shfl(mine, nl) + __shfl(mine, nl + 16)) + __shfl(mine, nl + 32);
                if (g == 0 && live) bits[p] = tot;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// rANS encode, one lane per row.  A workgroup is one wave owning 64 rows; the
// rows' (start, freq) words are staged through LDS in chunks of 64 symbols
// (coalesced reads, next chunk in flight while the current one is coded), so
// the serial chain per row never waits for memory.
// ---------------------------------------------------------------------------
constexpr int kRansRows = 64;
constexpr int kRansChunk = 64;
// Padding symbol (start 0, frequency 2^16): pushing it leaves the state unchanged
// and never renormalises, so every chunk can be coded as a full one.
constexpr uint32_t kRansNop = 0xFFFF0000u;

// 1/f in fp64 for 1 <= f < 2^17: hardware estimate plus two Newton steps
// (relative error ~2^-52).  Independent of the coder state, so several of these
// are computed ahead of the serial chain.
__device__ __forceinline__ double rans_recip(uint32_t f32) {
    const double fd = (double)f32;
    double rf = __builtin_amdgcn_rcp(fd);
    rf = __builtin_fma(__builtin_fma(-fd, rf, 1.0), rf, rf);
    rf = __builtin_fma(__builtin_fma(-fd, rf, 1.0), rf, rf);
    return rf;
}

// x <- C(x, (start, f)) with an exact x / f for x < 2^47 * f: the fp64 quotient
// estimate is within one of the truth, so the remainder x - q f lies in (-f, 2f)
// and its low 32 bits decide the correction.  Branch-free.
__device__ __forceinline__ void rans_push(uint64_t& x, uint32_t f, uint32_t start, double rf) {
    const double xd = __builtin_fma((double)(uint32_t)(x >> 32), 4294967296.0, (double)(uint32_t)x);
    // round(xd * rf) read off the mantissa after adding 2^52 (the quotient is below 2^47)
    const double qd = __builtin_fma(xd, rf, 4503599627370496.0);
    uint64_t q = (uint64_t)__double_as_longlong(qd) & 0x000FFFFFFFFFFFFFull;
    int32_t rem = (int32_t)((uint32_t)x - (uint32_t)q * f);
    const int32_t neg = rem < 0 ? 1 : 0, over = rem >= (int32_t)f ? 1 : 0;
    rem += neg ? (int32_t)f : 0;
    rem -= over ? (int32_t)f : 0;
    q += (uint64_t)(int64_t)(over - neg);
    x = (q << 16) + (uint64_t)((uint32_t)rem + start);
}

__global__ void __launch_bounds__(kRansRows)
rans_rows_kernel(const uint32_t* __restrict__ sf, int W, uint32_t rows, uint32_t* __restrict__ slabs,
                 uint32_t* __restrict__ row_words) {
    __shared__ uint32_t buf[2][kRansRows][kRansChunk + 1];
    const int lane = threadIdx.x;
    const uint32_t row0 = blockIdx.x * kRansRows;
    const uint32_t row = row0 + lane;
    const uint32_t nsym = 3u * (uint32_t)W;
    const int nchunks = (int)((nsym + kRansChunk - 1) / kRansChunk);
    const uint32_t live_rows = min((uint32_t)kRansRows, rows - row0);
    const size_t sw = slab_words(W);
    uint32_t* slab = slabs + (size_t)min(row, rows - 1) * sw;
    size_t wp = sw;
    uint64_t x = kRansL;

    uint32_t pre[kRansRows];   // chunk being fetched: element r is symbol k*64 + lane of row row0 + r
    auto fetch = [&](int k) {
        const uint32_t idx = (uint32_t)k * kRansChunk + lane;
#pragma unroll
        for (int r = 0; r < kRansRows; ++r)
            pre[r] = ((uint32_t)r < live_rows && idx < nsym) ? sf[(size_t)(row0 + r) * nsym + idx] : kRansNop;
    };
    auto stage = [&](int b) {
#pragma unroll
        for (int r = 0; r < kRansRows; ++r) buf[b][r][lane] = pre[r];
    };
    fetch(nchunks - 1);
    stage((nchunks - 1) & 1);
    __syncthreads();
    for (int k = nchunks - 1; k >= 0; --k) {
        if (k > 0) fetch(k - 1);
        if (row < rows) {
            constexpr int kU = 8;   // reciprocals of the next 8 symbols are computed side by side
            for (int i0 = kRansChunk; i0 > 0; i0 -= kU) {
                uint32_t v[kU];
                double rf[kU];
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    v[u] = buf[k & 1][lane][i0 - 1 - u];
                    rf[u] = rans_recip((v[u] >> 16) + 1u);
                }
                // scheduling only: the eight reciprocals are finished before the serial chain starts
                asm volatile("" : "+v"(rf[0]), "+v"(rf[1]), "+v"(rf[2]), "+v"(rf[3]), "+v"(rf[4]), "+v"(rf[5]), "+v"(rf[6]), "+v"(rf[7]));
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    const uint32_t start = v[u] & 0xFFFFu, f = (v[u] >> 16) + 1u;
                    // renormalise when x >= f * 2^47; the word is stored either way and only
                    // kept (wp moves) when it was due: no branch on the serial chain
                    const bool emit = (uint32_t)(x >> 47) >= f;
                    slab[wp - 1] = (uint32_t)x;
                    wp -= emit ? 1 : 0;
                    x = emit ? (x >> 32) : x;
                    rans_push(x, f, start, rf[u]);
                }
            }
        }
        if (k > 0) stage((k - 1) & 1);
        __syncthreads();
    }
    if (row < rows) {
        slab[--wp] = (uint32_t)(x >> 32);
        slab[--wp] = (uint32_t)x;
        row_words[row] = (uint32_t)(sw - wp);
    }
}

// Single workgroup: offsets[k] = 4 * sum_{j<k} row_words[j]; header; total size.
__global__ void __launch_bounds__(1024)
scan_kernel(const uint32_t* __restrict__ row_words, uint32_t rows, int n, int H, int W, uint32_t dist,
            uint8_t* __restrict__ stream, uint64_t* __restrict__ total_bytes) {
    __shared__ uint64_t part[1024];
    __shared__ uint64_t carry;
    uint64_t* offsets = reinterpret_cast<uint64_t*>(stream + kStreamHeader);
    if (threadIdx.x == 0) {
        carry = 0;
        uint32_t* hdr = reinterpret_cast<uint32_t*>(stream);
        hdr[0] = kStreamMagic; hdr[1] = 1; hdr[2] = (uint32_t)n; hdr[3] = (uint32_t)H; hdr[4] = (uint32_t)W;
        hdr[5] = kModelTag; hdr[6] = dist; hdr[7] = 0;
    }
    __syncthreads();
    for (uint32_t base = 0; base < rows; base += 1024) {
        const uint32_t k = base + threadIdx.x;
        const uint64_t mine = k < rows ? 4ull * row_words[k] : 0ull;
        part[threadIdx.x] = mine;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            const uint64_t add = threadIdx.x >= (uint32_t)d ? part[threadIdx.x - d] : 0ull;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        if (k < rows) offsets[k] = carry + part[threadIdx.x] - mine;
        __syncthreads();
        if (threadIdx.x == 1023) carry += part[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        offsets[rows] = carry;
        *total_bytes = (uint64_t)kStreamHeader + 8ull * (rows + 1) + carry;
    }
}

__global__ void __launch_bounds__(64)
compact_kernel(const uint32_t* __restrict__ slabs, const uint32_t* __restrict__ row_words, int W, uint32_t rows,
               uint8_t* __restrict__ stream, uint64_t cap_bytes, int* status) {
    const uint32_t row = blockIdx.x;
    const size_t sw = slab_words(W);
    const uint64_t table = (uint64_t)kStreamHeader + 8ull * (rows + 1);
    const uint64_t off = reinterpret_cast<const uint64_t*>(stream + kStreamHeader)[row];
    const uint32_t nw = row_words[row];
    if (table + off + 4ull * nw > cap_bytes) {
        if (threadIdx.x == 0) set_error(status, PCC_E_CAP);
        return;
    }
    const uint32_t* src = slabs + (size_t)row * sw + (sw - nw);
    uint32_t* dst = reinterpret_cast<uint32_t*>(stream + table + off);
    for (uint32_t i = threadIdx.x; i < nw; i += blockDim.x) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// wavefront decode
//
// One workgroup of 4 waves owns a band of 16 image rows; step t decodes pixel
// (r, t - 2r) of each row.  Per step:
//   network   the 16 pixels form one MFMA tile; each wave computes a quarter
//             of every layer's out-blocks with its weight slices held in
//             registers for the whole kernel, and the layers meet in LDS
//   search    16 lanes per pixel find the symbol with two 16-way rounds of
//             Cq evaluations per channel (R, then G given R, then B given R,G)
//   publish   the pixel goes to the LDS ring (next steps' neighbourhoods), to
//             the output image and, for the band's last two rows, to a mailbox
//             in global memory that the band below polls
// ---------------------------------------------------------------------------
#ifdef PCC_PHASE_TIMING
// Tuning aid (off in normal builds): cycles spent per phase of a decode step,
// accumulated by thread 0 of the band holding ticket 1 (or 0 if there is one band).
__device__ unsigned long long g_phase_cycles[16];
#define PCC_PHASE(k) do { if (timed) { const unsigned long long now_ = clock64(); phase_acc[k] += now_ - phase_t; phase_t = now_; } } while (0)
#else
#define PCC_PHASE(k) do { } while (0)
#endif
constexpr int kDecThreads = 256;
constexpr int kActBytes = 5 * 2 * 64 * 16;                     // one layer's activations: [k-block][hi,lo][lane][16 B]
// decode LDS: the normal-CDF table, two activation buffers, head outputs, mixtures, ring
constexpr int kDLutOff = 0;
constexpr int kDAct0Off = (kLutEntries + 1) * 8;               // 12,304
constexpr int kDAct1Off = kDAct0Off + kActBytes;
constexpr int kDHeadOff = kDAct1Off + kActBytes;               // [16 pixels][4 groups][16] fp32, (group, register) layout
constexpr int kDCpOff = kDHeadOff + 16 * 64 * 4;               // [16 pixels][3 channels][16] fp32: pi[5], mu[5], a[5], pad
// Ring of recently decoded pixels as first-layer inputs: [18 rows][16 columns][3] bf16.
// Rows 0,1 are the two rows above the band.  Column c lives at slots c & 7 and
// (c & 7) + 8, so the twelve values of columns c-2..c+1 are always contiguous.
constexpr int kRingRowElems = 16 * 3;
constexpr int kDRingOff = kDCpOff + 16 * 3 * 16 * 4;
constexpr int kDMiscOff = kDRingOff + 18 * kRingRowElems * 2;  // ticket, abort flag
constexpr int kDecLdsBytes = kDMiscOff + 64;
static_assert(kDAct0Off % 16 == 0 && kDCpOff % 16 == 0, "vector alignment");

// All-reduce over the 16 lanes of a DPP row by rotations.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_row(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t row_allmax(uint32_t v) {
    v = max(v, dpp_row<0x121>(v)); v = max(v, dpp_row<0x122>(v));
    v = max(v, dpp_row<0x124>(v)); v = max(v, dpp_row<0x128>(v));
    return v;
}
__device__ __forceinline__ uint32_t row_allmin(uint32_t v) {
    v = min(v, dpp_row<0x121>(v)); v = min(v, dpp_row<0x122>(v));
    v = min(v, dpp_row<0x124>(v)); v = min(v, dpp_row<0x128>(v));
    return v;
}

// rANS reader of one row, replicated in the 16 lanes of the pixel's group.  The
// next 32 stream words sit in registers, lane j holding words base+j and
// base+16+j, so a renormalisation never waits for memory: the refill issued
// when a 16-word block is used up is not needed for another 16 words.
struct RowReader {
    uint64_t x;
    const uint32_t* words;  // payload after the 8-byte state
    uint32_t nwords, pos;   // pos: words consumed so far
    uint32_t cur, nxt;      // words[(pos & ~15) + j], words[(pos & ~15) + 16 + j]
    bool bad;
};

__device__ __forceinline__ void reader_init(RowReader& rd, const uint32_t* payload, uint32_t nwords_total, int j) {
    rd.x = (uint64_t)payload[0] | ((uint64_t)payload[1] << 32);
    rd.words = payload + 2;
    rd.nwords = nwords_total - 2;
    rd.pos = 0;
    rd.cur = (uint32_t)j < rd.nwords ? rd.words[j] : 0u;
    rd.nxt = (uint32_t)j + 16u < rd.nwords ? rd.words[j + 16] : 0u;
    rd.bad = false;
    if (rd.x < kRansL || (rd.x >> 63)) { rd.bad = true; rd.x = kRansL; }
}

__device__ __forceinline__ void reader_advance(RowReader& rd, uint32_t slot, uint32_t start, uint32_t freq, int j,
                                               bool active) {
    const uint32_t w = row_allmax((uint32_t)j == (rd.pos & 15u) ? rd.cur : 0u);   // words[pos], in every lane of the group
    const uint64_t x1 = (uint64_t)freq * (rd.x >> 16) + slot - start;
    const bool renorm = active && x1 < kRansL;
    if (active) rd.x = renorm ? ((x1 << 32) | w) : x1;
    if (renorm) {
        if (rd.pos >= rd.nwords) rd.bad = true;
        rd.pos += 1;
        if ((rd.pos & 15u) == 0u) {
            rd.cur = rd.nxt;
            const uint32_t idx = rd.pos + 16u + (uint32_t)j;
            rd.nxt = idx < rd.nwords ? rd.words[idx] : 0u;
        }
    }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for
// every outstanding global access (pixel stores, mailbox traffic, stream-word and
// mailbox prefetches), which would put HBM latency on the step's critical path
// five times per step; nothing here hands global data from thread to thread.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// This wave's weight slices of one layer: out-blocks ob = wave + 4 s.  Where the
// wave has no such block (ob >= NOB) it holds a copy of the layer's last block
// and its results are discarded.
template <int NOB, int NKB, int SLOTS>
struct WaveLayer {
    u32x4_t a[SLOTS][NKB];
    f32x4_t bias[SLOTS];
    __device__ __forceinline__ void load(const uint8_t* __restrict__ w, const float* __restrict__ b, int lane, int wave) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int ob = min(wave + 4 * s, NOB - 1);
            bias[s] = *reinterpret_cast<const f32x4_t*>(b + 16 * ob + 4 * (lane >> 4));
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
                a[s][kb] = *reinterpret_cast<const u32x4_t*>(w + ((ob * NKB + kb) * 64 + lane) * 16);
        }
    }
};

// One hidden layer on this wave's out-blocks.  Same arithmetic per output element
// as hidden_layer<> in pcc_device.h: bias, then k-blocks in order, each hi then
// lo; ReLU; split into hi + lo.
template <int NOB, int NKB, int SLOTS, bool SPLIT_IN>
__device__ __forceinline__ void dec_hidden_layer(const WaveLayer<NOB, NKB, SLOTS>& wl, int lane, int wave,
                                                 const u32x4_t (&in)[NKB][2], uint8_t* __restrict__ act_out) {
    f32x4_t acc[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) acc[s] = wl.bias[s];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) acc[s] = mfma16(wl.a[s][kb], in[kb][0], acc[s]);
        if (SPLIT_IN) {
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) acc[s] = mfma16(wl.a[s][kb], in[kb][1], acc[s]);
        }
    }
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int ob = wave + 4 * s;
        if (ob < NOB) {
            uint32_t l0, l1;
            const uint32_t h0 = relu_split_bf16(acc[s].x, acc[s].y, l0);
            const uint32_t h1 = relu_split_bf16(acc[s].z, acc[s].w, l1);
            // out-block ob is half (ob & 1) of k-block ob/2 of the next layer's operand
            uint8_t* dst = act_out + (((ob >> 1) * 2) * 64 + lane) * 16 + 8 * (ob & 1);
            *reinterpret_cast<uint2*>(dst) = make_uint2(h0, h1);
            *reinterpret_cast<uint2*>(dst + 64 * 16) = make_uint2(l0, l1);
        }
    }
}

template <int NKB>
__device__ __forceinline__ void dec_load_act(const uint8_t* __restrict__ act, int lane, u32x4_t (&in)[NKB][2]) {
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        in[kb][0] = *reinterpret_cast<const u32x4_t*>(act + ((kb * 2 + 0) * 64 + lane) * 16);
        in[kb][1] = *reinterpret_cast<const u32x4_t*>(act + ((kb * 2 + 1) * 64 + lane) * 16);
    }
}

// Symbol search by the 16 lanes (j = 0..15) of one pixel: two rounds of 16
// evaluations.  All lanes of the group return the same x, start, freq.
__device__ __forceinline__ int group_search(const ChanParams& cp, uint32_t slot, const float2* __restrict__ lut, int lane,
                                            uint32_t& start, uint32_t& freq) {
    const int j = lane & 15, shift = lane & 48;
    // round 1: Cq(16 j); lanes 0..b satisfy Cq <= slot (Cq is increasing and Cq(0) = 0)
    const uint32_t c1 = j == 0 ? 0u : cq_eval(cp, 16 * j, lut);
    const bool p1 = c1 <= slot;
    const int b = __popcll((__ballot(p1) >> shift) & 0xFFFFull) - 1;
    const uint32_t lo1 = row_allmax(p1 ? c1 : 0u);           // Cq(16 b)
    const uint32_t hi1 = row_allmin(p1 ? 65536u : c1);       // Cq(16 b + 16)
    // round 2: Cq(16 b + j)
    const uint32_t c2 = j == 0 ? lo1 : cq_eval(cp, 16 * b + j, lut);
    const bool p2 = c2 <= slot;
    const int cnt2 = __popcll((__ballot(p2) >> shift) & 0xFFFFull);
    start = row_allmax(p2 ? c2 : 0u);
    freq = row_allmin(p2 ? hi1 : c2) - start;
    return 16 * b + cnt2 - 1;
}

// MINBLOCKS = 1: all registers to one workgroup per CU (lowest latency per step; used when
// every band gets a CU of its own).  MINBLOCKS = 2: two workgroups share a CU (a few
// spills, ~15 % slower per step, but the second band fills the first one's stalls; used
// when there are more bands than CUs).
template <int MINBLOCKS>
__global__ void __launch_bounds__(kDecThreads, MINBLOCKS)
decode_kernel(const uint8_t* __restrict__ model, const uint8_t* __restrict__ stream, uint64_t nbytes, int n, int H,
              int W, int nbands, uint32_t dist, uint8_t* __restrict__ img_out, uint32_t* mailbox, int* status,
              uint32_t spin_limit) {
    extern __shared__ __align__(16) uint8_t lds[];
    float2* lut = reinterpret_cast<float2*>(lds + kDLutOff);
    uint8_t* act0 = lds + kDAct0Off;
    uint8_t* act1 = lds + kDAct1Off;
    float* headout = reinterpret_cast<float*>(lds + kDHeadOff);
    float* cpbuf = reinterpret_cast<float*>(lds + kDCpOff);
    uint16_t* ring = reinterpret_cast<uint16_t*>(lds + kDRingOff);   // [18][16][3] bf16
    int* misc = reinterpret_cast<int*>(lds + kDMiscOff);            // [0] ticket, [1] abort
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // network role: pixel nl of the tile, k-slot group g
    const int g = lane >> 4, nl = lane & 15;
    // search role: pixel q of the band, lane j of its group
    const int q = 4 * wave + (lane >> 4), j = lane & 15;

    // Bands take tickets in start order: a band only ever waits for the band
    // above it, which holds a smaller ticket and is therefore already running.
    if (tid == 0) { misc[0] = atomicAdd(&status[kStTicket], 1); misc[1] = 0; }
    {
        const float2* src = reinterpret_cast<const float2*>(model + kLutOff);
        for (int i = tid; i < kLutEntries + 1; i += kDecThreads) lut[i] = src[i];
    }
    for (int i = tid; i < 18 * kRingRowElems; i += kDecThreads) ring[i] = 0;

    // this wave's weights stay in registers
    WaveLayer<kL1_OB, kL1_KB, 3> wl1;
    WaveLayer<kL2_OB, kL2_KB, 3> wl2;
    WaveLayer<kL3_OB, kL3_KB, 2> wl3;
    WaveLayer<kL4_OB, kL4_KB, 1> wl4;
    wl1.load(model + kW1Off, reinterpret_cast<const float*>(model + kB1Off), lane, wave);
    wl2.load(model + kW2Off, reinterpret_cast<const float*>(model + kB2Off), lane, wave);
    wl3.load(model + kW3Off, reinterpret_cast<const float*>(model + kB3Off), lane, wave);
    wl4.load(model + kW4Off, reinterpret_cast<const float*>(model + kB4Off), lane, wave);
    __syncthreads();

    const int ticket = misc[0];
    const int im = ticket / nbands, band = ticket - im * nbands;
    if (im >= n) return;
    const float lut_scale = *reinterpret_cast<const float*>(model + kLutScaleOff);

    const int r0 = band * kBandRows;
    const uint64_t rows_total = (uint64_t)n * H;
    const uint64_t table = (uint64_t)kStreamHeader + 8ull * (rows_total + 1);
    const uint64_t payload_bytes = nbytes - table;   // host guarantees nbytes >= table

    if (ticket == 0 && tid == 0) {
        const uint32_t* hdr = reinterpret_cast<const uint32_t*>(stream);
        const uint64_t last = reinterpret_cast<const uint64_t*>(stream + kStreamHeader)[rows_total];
        if (hdr[0] != kStreamMagic || hdr[1] != 1u || hdr[2] != (uint32_t)n || hdr[3] != (uint32_t)H ||
            hdr[4] != (uint32_t)W || hdr[5] != kModelTag || hdr[6] != dist || last != payload_bytes)
            set_error(status, PCC_E_STREAM);
    }

    // search role: row of this lane's pixel and its stream reader (the same in all 16 lanes of the group)
    const int qrow = r0 + q;
    const bool qrow_ok = qrow < H;
    RowReader rd;
    rd.x = kRansL; rd.words = nullptr; rd.nwords = 0; rd.pos = 0; rd.cur = 0; rd.nxt = 0; rd.bad = false;
    if (qrow_ok) {
        const uint64_t* offs = reinterpret_cast<const uint64_t*>(stream + kStreamHeader);
        const uint64_t rowg = (uint64_t)im * H + qrow;
        const uint64_t a = offs[rowg], b = offs[rowg + 1];
        if (a > b || b > payload_bytes || (b - a) < 8 || ((b - a) & 3) != 0 || (a & 3) != 0 ||
            (b - a) > 4ull * slab_words(W))
            rd.bad = true;
        else
            reader_init(rd, reinterpret_cast<const uint32_t*>(stream + table + a), (uint32_t)((b - a) / 4), j);
    }

    uint8_t* out_img = img_out + (size_t)im * H * W * 3;
    const uint32_t* mail_in = mailbox + ((size_t)im * nbands + (band > 0 ? band - 1 : 0)) * 2 * (size_t)W;
    uint32_t* mail_out = mailbox + ((size_t)im * nbands + band) * 2 * (size_t)W;

    const int last_row = min(r0 + kBandRows - 1, H - 1);
    const int t_begin = 2 * r0, t_end = 2 * last_row + W - 1;
    const bool fetcher = band > 0 && tid < 2;     // thread 0: row r0-2 -> ring row 0; thread 1: row r0-1 -> ring row 1
    const uint32_t* mail_row = mail_in + (size_t)(tid & 1) * W;
    uint32_t pf = 0;                              // mailbox word for the next column, requested a step early

    // bf16 of the three channels of pixel word px into both copies of column cc of a ring row
    auto ring_put = [&](int rrow, int cc, uint32_t px) {
        uint16_t* d = ring + rrow * kRingRowElems + (cc & 7) * 3;
        const uint16_t v0 = (uint16_t)byte_to_bf16(px & 0xFFu), v1 = (uint16_t)byte_to_bf16((px >> 8) & 0xFFu),
                       v2 = (uint16_t)byte_to_bf16((px >> 16) & 0xFFu);
        d[0] = v0; d[1] = v1; d[2] = v2;
        d[24] = v0; d[25] = v1; d[26] = v2;
    };
    // Bring columns 0 and 1 of the two rows above the band into the ring, then keep
    // one column ahead: the step at t needs column (t - t_begin) + 1.
    auto fetch_column = [&](int cc, uint32_t have) -> bool {   // returns false on abort
        uint32_t v = have, spins = 0;
        while (!(v & kMailTag)) {
            v = __hip_atomic_load(mail_row + cc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v & kMailTag) break;
            ++spins;
            if (spins > spin_limit) { set_error(status, PCC_E_INTERNAL); return false; }
            if ((spins & 63u) == 0u &&
                __hip_atomic_load(&status[kStAbort], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
                return false;
            __builtin_amdgcn_s_sleep(1);
        }
        ring_put(tid & 1, cc, v);
        return true;
    };
    if (fetcher) {
        bool ok = fetch_column(0, 0u);
        if (ok && W > 1) ok = fetch_column(1, 0u);
        if (ok && W > 2) pf = __hip_atomic_load(mail_row + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!ok) {
            __hip_atomic_store(&status[kStAbort], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            misc[1] = 1;
        }
    }
    lds_barrier();

    // network role: this lane's eight first-layer inputs are two runs of four
    // consecutive ring values (row, offset within the 12-value window of columns c-2..c+1)
    const int gA_row = nl + (g >= 2 ? 1 : 0), gA_off = (g & 1) ? 8 : 0;
    const int gB_row = nl + (g == 0 ? 0 : (g == 2 ? 1 : 2)), gB_off = (g == 1) ? 0 : 4;
    const uint16_t* gA = ring + gA_row * kRingRowElems + gA_off;
    const uint16_t* gB = ring + gB_row * kRingRowElems + gB_off;

#ifdef PCC_PHASE_TIMING
    const bool timed = tid == 0 && ticket == (nbands * n > 1 ? 1 : 0);
    unsigned long long phase_acc[16] = {};
    unsigned long long phase_t = clock64();
#endif
    for (int t = t_begin; t <= t_end; ++t) {
        if ((t & 7) == 0 && misc[1] != 0) break;  // uniform: written before the last barrier; a late exit only decodes garbage
        PCC_PHASE(15);

        // ---- gather C_ij from the ring (zeros stand for pixels outside the image); every wave builds the full tile
        u32x4_t in1[1][2];
        {
            const int c = t - 2 * (r0 + nl);
            const int w0 = ((c - 2) & 7) * 3;
            uint32_t v[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] = gA[w0 + i]; v[4 + i] = gB[w0 + i]; }
            // one batch of LDS reads
            asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]));
            in1[0][0].x = v[0] | (v[1] << 16);
            in1[0][0].y = v[2] | (v[3] << 16);
            in1[0][0].z = v[4] | (v[5] << 16);
            in1[0][0].w = v[6] | (v[7] << 16);
            in1[0][1] = in1[0][0];   // unused (layer-1 inputs are exact)
        }
        PCC_PHASE(0);

        // ---- network, layers meeting in LDS
        dec_hidden_layer<kL1_OB, kL1_KB, 3, false>(wl1, lane, wave, in1, act0);
        lds_barrier();
        PCC_PHASE(1);
        {
            u32x4_t in[kL2_KB][2];
            dec_load_act<kL2_KB>(act0, lane, in);
            dec_hidden_layer<kL2_OB, kL2_KB, 3, true>(wl2, lane, wave, in, act1);
        }
        lds_barrier();
        PCC_PHASE(2);
        {
            u32x4_t in[kL3_KB][2];
            dec_load_act<kL3_KB>(act1, lane, in);
            dec_hidden_layer<kL3_OB, kL3_KB, 2, true>(wl3, lane, wave, in, act0);
        }
        lds_barrier();
        PCC_PHASE(3);
        {
            u32x4_t in[kL4_KB][2];
            dec_load_act<kL4_KB>(act0, lane, in);
            f32x4_t acc = wl4.bias[0];
#pragma unroll
            for (int kb = 0; kb < kL4_KB; ++kb) {
                acc = mfma16(wl4.a[0][kb], in[kb][0], acc);
                acc = mfma16(wl4.a[0][kb], in[kb][1], acc);
            }
            // registers s = 4 wave + i of group g, kept in (group, register) order
            *reinterpret_cast<f32x4_t*>(headout + nl * 64 + g * 16 + 4 * wave) = acc;
        }
        lds_barrier();
        PCC_PHASE(4);

        // ---- mixtures: lane j < 15 of pixel q prepares component j % 5 of channel j / 5
        if (j < 15) {
            const int ch = j / 5, k = j - 5 * ch;
            const f32x4_t* src = reinterpret_cast<const f32x4_t*>(headout + q * 64 + ch * 16);
            const f32x4_t v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];
            const float raw[15] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w, v2.x, v2.y, v2.z, v2.w, v3.x, v3.y, v3.z};
            ChanParams all;
            channel_setup(raw, lut_scale, all);
            float pk = all.pi[0], mk = all.mu[0], ak = all.a[0];
#pragma unroll
            for (int kk = 1; kk < 5; ++kk) if (k == kk) { pk = all.pi[kk]; mk = all.mu[kk]; ak = all.a[kk]; }
            float* dst = cpbuf + (q * 3 + ch) * 16 + k;
            dst[0] = pk; dst[5] = mk; dst[10] = ak;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");

        // everything the three searches need, in one batch of LDS reads
        ChanParams cpr, cpg, cpb;
        float alpha[5], beta[5], gamma[5];
        {
            auto load_cp = [&](int ch, ChanParams& cp) {
                const f32x4_t* src = reinterpret_cast<const f32x4_t*>(cpbuf + (q * 3 + ch) * 16);
                const f32x4_t v0 = src[0], v1 = src[1], v2 = src[2], v3 = src[3];
                cp.pi[0] = v0.x; cp.pi[1] = v0.y; cp.pi[2] = v0.z; cp.pi[3] = v0.w; cp.pi[4] = v1.x;
                cp.mu[0] = v1.y; cp.mu[1] = v1.z; cp.mu[2] = v1.w; cp.mu[3] = v2.x; cp.mu[4] = v2.y;
                cp.a[0] = v2.z; cp.a[1] = v2.w; cp.a[2] = v3.x; cp.a[3] = v3.y; cp.a[4] = v3.z;
            };
            load_cp(0, cpr); load_cp(1, cpg); load_cp(2, cpb);
            const float* hq = headout + q * 64;
            const f32x4_t* g3 = reinterpret_cast<const f32x4_t*>(hq + 48);
            const f32x4_t c0 = g3[0], c1 = g3[1], c2 = g3[2];
            alpha[0] = hq[16 + 15]; alpha[1] = c0.x; alpha[2] = c0.y; alpha[3] = c0.z; alpha[4] = c0.w;
            beta[0] = hq[32 + 15]; beta[1] = c1.x; beta[2] = c1.y; beta[3] = c1.z; beta[4] = c1.w;
            gamma[0] = c2.x; gamma[1] = c2.y; gamma[2] = c2.z; gamma[3] = c2.w; gamma[4] = hq[48 + 12];
        }
        PCC_PHASE(5);

        const int c = t - 2 * qrow;
        const bool active = qrow_ok && c >= 0 && c < W;
        uint32_t start, freq;
        // R
        uint32_t slot = (uint32_t)rd.x & 0xFFFFu;
        const int sr = group_search(cpr, slot, lut, lane, start, freq);
        reader_advance(rd, slot, start, freq, j, active);
        const float rhat = (float)sr * (1.0f / 256.0f);
        PCC_PHASE(6);
        // G given R
        couple_green(cpg, alpha, rhat);
        slot = (uint32_t)rd.x & 0xFFFFu;
        const int sg = group_search(cpg, slot, lut, lane, start, freq);
        reader_advance(rd, slot, start, freq, j, active);
        const float ghat = (float)sg * (1.0f / 256.0f);
        PCC_PHASE(7);
        // B given R, G
        couple_blue(cpb, beta, gamma, rhat, ghat);
        slot = (uint32_t)rd.x & 0xFFFFu;
        const int sb = group_search(cpb, slot, lut, lane, start, freq);
        reader_advance(rd, slot, start, freq, j, active);
        PCC_PHASE(8);

        // ---- publish
        if (j == 0 && active) {
            const uint32_t px = (uint32_t)sr | ((uint32_t)sg << 8) | ((uint32_t)sb << 16);
            ring_put(q + 2, c, px);
            if (c == W - 1) ring_put(q + 2, W, 0u);   // the column right of the image reads as zero
            uint8_t* o = out_img + ((size_t)qrow * W + c) * 3;
            o[0] = (uint8_t)sr; o[1] = (uint8_t)sg; o[2] = (uint8_t)sb;
            if (q >= kBandRows - 2)
                __hip_atomic_store(mail_out + (size_t)(q - (kBandRows - 2)) * W + c, px | kMailTag, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if (c == W - 1 && (rd.bad || rd.x != kRansL || rd.pos != rd.nwords)) set_error(status, PCC_E_STREAM);
        }
        // ---- rows above the band: column needed by the next step, and request the one after
        if (fetcher) {
            const int cc = t - t_begin + 2;
            if (cc == W) ring_put(tid & 1, W, 0u);    // the column right of the image reads as zero
            if (cc < W && t < t_end) {
                if (!fetch_column(cc, pf)) {
                    __hip_atomic_store(&status[kStAbort], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    misc[1] = 1;
                }
                pf = (cc + 1 < W) ? __hip_atomic_load(mail_row + cc + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
            }
        }
        PCC_PHASE(9);
        lds_barrier();
        PCC_PHASE(10);
    }
#ifdef PCC_PHASE_TIMING
    if (timed) for (int k = 0; k < 16; ++k) g_phase_cycles[k] = phase_acc[k];
#endif
}

// ---------------------------------------------------------------------------
// test hook: full tables from given head outputs
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
cdf_tables_kernel(const uint8_t* __restrict__ model, const float* __restrict__ params, const uint8_t* __restrict__ rg,
                  size_t count, uint32_t* __restrict__ cq) {
    extern __shared__ __align__(16) uint8_t lds[];
    float2* lut = reinterpret_cast<float2*>(lds);
    const float2* src = reinterpret_cast<const float2*>(model + kLutOff);
    for (int i = threadIdx.x; i < kLutEntries + 1; i += blockDim.x) lut[i] = src[i];
    __syncthreads();
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= count * 3) return;
    const size_t p = idx / 3;
    const int ch = (int)(idx - p * 3);
    const float* o = params + p * PCC_HEAD_OUTPUTS;
    float raw[15];
    for (int s = 0; s < 15; ++s) raw[s] = o[15 * ch + s];
    ChanParams cp;
    channel_setup(raw, *reinterpret_cast<const float*>(model + kLutScaleOff), cp);
    const float rhat = (float)rg[2 * p] * (1.0f / 256.0f), ghat = (float)rg[2 * p + 1] * (1.0f / 256.0f);
    float c1[5], c2[5];
    for (int k = 0; k < 5; ++k) { c1[k] = ch == 1 ? o[45 + k] : o[50 + k]; c2[k] = o[55 + k]; }
    if (ch == 1) couple_green(cp, c1, rhat);
    if (ch == 2) couple_blue(cp, c1, c2, rhat, ghat);
    uint32_t* dst = cq + idx * 257;
    for (int e = 0; e <= 256; ++e) dst[e] = cq_full(cp, e, lut);
}

}  // namespace pcc

// ===========================================================================
// host side
// ===========================================================================
using namespace pcc;

struct pcc_ctx {
    int device = 0;
    uint8_t* d_model = nullptr;
    // workspace (grown on demand)
    uint8_t* d_ws = nullptr;
    size_t ws_bytes = 0;
    int* d_status = nullptr;       // kStWords ints
    uint64_t* d_total = nullptr;
    int* h_status = nullptr;       // pinned, kStWords ints + 2 for the total
    // layout of the last encode inside the workspace
    uint32_t* d_sf = nullptr;
    size_t sf_count = 0;
    int num_cus = 0;
    uint32_t dist = 0;             // written to / checked against stream header word 6
    int encode_variant = kDefaultEncodeVariant;
    // optional per-kernel timing
    bool profiling = false;
    hipEvent_t ev[2 * PCC_N_TIMINGS] = {};
    bool ev_used[PCC_N_TIMINGS] = {};
    float last_ms[PCC_N_TIMINGS] = {};
};

namespace {

inline uint32_t rd32(const uint8_t* p) {
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
inline float rdf(const uint8_t* p) { uint32_t u = rd32(p); float f; memcpy(&f, &u, 4); return f; }

// fp32 -> bf16 bits, exact values only (caller has checked representability)
inline bool bf16_exact(float f, uint16_t* out) {
    uint32_t u; memcpy(&u, &f, 4);
    *out = (uint16_t)(u >> 16);
    return (u & 0xFFFFu) == 0u;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

int ensure_workspace(pcc_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return PCC_OK;
    if (ctx->d_ws) { (void)hipFree(ctx->d_ws); ctx->d_ws = nullptr; ctx->ws_bytes = 0; }
    ctx->d_sf = nullptr; ctx->sf_count = 0;
    const size_t want = bytes + bytes / 8 + 4096;
    if (hipMalloc((void**)&ctx->d_ws, want) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    ctx->ws_bytes = want;
    return PCC_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline void prof_reset(pcc_ctx* ctx) {
    for (int i = 0; i < PCC_N_TIMINGS; ++i) { ctx->ev_used[i] = false; ctx->last_ms[i] = 0.0f; }
}
inline void prof_begin(pcc_ctx* ctx, int which, hipStream_t st) {
    if (ctx->profiling) (void)hipEventRecord(ctx->ev[2 * which], st);
}
inline void prof_end(pcc_ctx* ctx, int which, hipStream_t st) {
    if (ctx->profiling) { (void)hipEventRecord(ctx->ev[2 * which + 1], st); ctx->ev_used[which] = true; }
}
// after the stream has been synchronised
inline void prof_collect(pcc_ctx* ctx) {
    if (!ctx->profiling) return;
    for (int i = 0; i < PCC_N_TIMINGS; ++i)
        if (ctx->ev_used[i] && hipEventElapsedTime(&ctx->last_ms[i], ctx->ev[2 * i], ctx->ev[2 * i + 1]) != hipSuccess) {
            (void)hipGetLastError();
            ctx->last_ms[i] = 0.0f;
        }
}

bool dims_ok(int n, int H, int W) {
    if (n < 1 || H < 1 || W < 1) return false;
    const uint64_t P = (uint64_t)n * H * W;
    return P < (1ull << 31) && (uint64_t)W < (1u << 24) && (uint64_t)n * H < (1ull << 31) &&
           (uint64_t)H * W * 3 < (1ull << 31);   // byte offsets within one image are 32-bit
}

}  // namespace

extern "C" {

const char* pcc_strerror(int code) {
    switch (code) {
        case PCC_OK: return "ok";
        case PCC_E_ARG: return "invalid argument";
        case PCC_E_BLOB: return "unsupported or malformed weight blob";
        case PCC_E_CAP: return "output capacity too small";
        case PCC_E_STREAM: return "malformed stream";
        case PCC_E_HIP: return "HIP runtime error";
        case PCC_E_INTERNAL: return "internal error (zero frequency or device wait expired)";
        case PCC_E_UNIMPL: return "not implemented";
        default: return "unknown error";
    }
}

size_t pcc_stream_bound(int n, int H, int W) {
    if (n < 1 || H < 1 || W < 1) return 0;
    const size_t rows = (size_t)n * H;
    return (size_t)kStreamHeader + 8 * (rows + 1) + rows * 4 * slab_words(W);
}

long pcc_wavefront_steps(int H, int W) { return (long)W + 2L * (H - 1); }

int pcc_create(pcc_ctx** out, const void* h_blob, size_t blob_bytes, int hip_device) {
    if (!out || !h_blob) return PCC_E_ARG;
    *out = nullptr;
    const uint8_t* p = (const uint8_t*)h_blob;
    static const int dims[5] = {30, 160, 160, 128, 60};
    if (blob_bytes < 64 || rd32(p) != kBlobMagic || rd32(p + 4) != 1u || rd32(p + 8) != 4u) return PCC_E_BLOB;
    for (int i = 0; i < 5; ++i) if (rd32(p + 12 + 4 * i) != (uint32_t)dims[i]) return PCC_E_BLOB;
    const uint32_t dist = rd32(p + 60);   // 0 = Gaussian mixture (Eq. (1)), 1 = logistic mixture (Eq. (8))
    if (rd32(p + 44) != 5u || rd32(p + 48) != 10u || rd32(p + 52) != 2u || rd32(p + 56) != 0u || dist > 1u)
        return PCC_E_BLOB;
    size_t need = 64;
    for (int l = 0; l < 4; ++l) need += 4 * ((size_t)dims[l] * dims[l + 1] + dims[l + 1]);
    if (blob_bytes != need) return PCC_E_BLOB;

    const uint8_t* wsrc[4];
    const uint8_t* bsrc[4];
    const uint8_t* q = p + 64;
    for (int l = 0; l < 4; ++l) {
        wsrc[l] = q; q += 4 * (size_t)dims[l] * dims[l + 1];
        bsrc[l] = q; q += 4 * (size_t)dims[l + 1];
    }
    auto Wat = [&](int l, int o, int i) { return rdf(wsrc[l] + 4 * ((size_t)o * dims[l] + i)); };
    auto Bat = [&](int l, int o) { return rdf(bsrc[l] + 4 * (size_t)o); };

    std::vector<uint8_t> image(kModelBytes, 0);
    uint16_t* w16 = reinterpret_cast<uint16_t*>(image.data());
    static const int nob[4] = {kL1_OB, kL2_OB, kL3_OB, kL4_OB}, nkb[4] = {kL1_KB, kL2_KB, kL3_KB, kL4_KB};
    static const int woff[4] = {kW1Off, kW2Off, kW3Off, kW4Off}, boff[4] = {kB1Off, kB2Off, kB3Off, kB4Off};
    for (int l = 0; l < 4; ++l) {
        for (int ob = 0; ob < nob[l]; ++ob)
            for (int kb = 0; kb < nkb[l]; ++kb)
                for (int lane = 0; lane < 64; ++lane)
                    for (int i = 0; i < 8; ++i) {
                        const int m = lane & 15, g = lane >> 4;
                        // output feature of A row m of this out-block
                        const int o = l < 3 ? 16 * ob + m : head_index(m >> 2, 4 * ob + (m & 3));
                        // input feature of k-slot (g, i) of this k-block
                        const int in = l == 0 ? in1_index(g, i) : 32 * kb + kslot_feature(g, i);
                        float v = 0.0f;
                        if (o >= 0 && o < dims[l + 1] && in >= 0 && in < dims[l]) v = Wat(l, o, in);
                        uint16_t h;
                        if (!bf16_exact(v, &h)) return PCC_E_BLOB;
                        if (l == 0 && v != 0.0f) {
                            // fold the 1/256 input scaling into the first layer: exact unless it underflows
                            const float s = v * (1.0f / 256.0f);
                            if (!bf16_exact(s, &h) || s * 256.0f != v) return PCC_E_BLOB;
                        }
                        w16[(woff[l] + (((ob * nkb[l] + kb) * 64 + lane) * 16)) / 2 + i] = h;
                    }
        float* b = reinterpret_cast<float*>(image.data() + boff[l]);
        const int padded = 16 * nob[l];
        for (int s = 0; s < padded; ++s) {
            const int ob = s >> 4, m = s & 15;
            const int o = l < 3 ? s : head_index(m >> 2, 4 * ob + (m & 3));
            b[s] = (o >= 0 && o < dims[l + 1]) ? Bat(l, o) : 0.0f;
        }
    }
    // Component CDF table in units of 2^-24 so that forward differences are exact in fp32.
    float* lut = reinterpret_cast<float*>(image.data() + kLutOff);
    const double lut_scale = dist == 0 ? (double)kLutScaleGaussian : (double)kLutScaleLogistic;
    *reinterpret_cast<float*>(image.data() + kLutScaleOff) = (float)lut_scale;
    std::vector<double> tq(kLutEntries + 1);
    for (int i = 0; i < kLutEntries; ++i) {
        const double z = (i - 768) / lut_scale;
        const double F = dist == 0 ? 0.5 * erfc(-z / sqrt(2.0)) : 1.0 / (1.0 + exp(-z));
        tq[i] = nearbyint(F * 16777216.0);
    }
    tq[0] = 0.0;
    tq[kLutEntries - 1] = 16777216.0;
    tq[kLutEntries] = tq[kLutEntries - 1];
    for (int i = 0; i < kLutEntries; ++i) {
        lut[2 * i] = (float)(tq[i] / 16777216.0);
        lut[2 * i + 1] = (float)((tq[i + 1] - tq[i]) / 16777216.0);
    }
    lut[2 * kLutEntries] = 1.0f;
    lut[2 * kLutEntries + 1] = 0.0f;

    DeviceGuard guard(hip_device);
    if (!guard.ok) { (void)hipGetLastError(); return PCC_E_HIP; }
    pcc_ctx* ctx = new (std::nothrow) pcc_ctx();
    if (!ctx) return PCC_E_INTERNAL;
    ctx->device = hip_device;
    ctx->dist = dist;
    hipDeviceProp_t prop;
    bool ok = hipGetDeviceProperties(&prop, hip_device) == hipSuccess;
    if (ok) ctx->num_cus = prop.multiProcessorCount;
    ok = ok && hipMalloc((void**)&ctx->d_model, kModelBytes) == hipSuccess;
    ok = ok && hipMalloc((void**)&ctx->d_status, kStWords * sizeof(int) + sizeof(uint64_t)) == hipSuccess;
    ok = ok && hipHostMalloc((void**)&ctx->h_status, kStWords * sizeof(int) + sizeof(uint64_t), hipHostMallocDefault) == hipSuccess;
    ok = ok && hipMemcpy(ctx->d_model, image.data(), kModelBytes, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<1, 512>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kModelBytes) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<2, 512>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kModelBytes) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<1, 1024>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kModelBytes) == hipSuccess;
    if (const char* e = getenv("PCC_ENCODE_VARIANT")) {
        const int v = atoi(e);
        if (v >= 0 && v < 3) ctx->encode_variant = v;
    }
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kDecLdsBytes) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<2>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kDecLdsBytes) == hipSuccess;
    if (!ok) { (void)hipGetLastError(); pcc_destroy(ctx); return PCC_E_HIP; }
    ctx->d_total = reinterpret_cast<uint64_t*>(ctx->d_status + kStWords);
    *out = ctx;
    return PCC_OK;
}

void pcc_destroy(pcc_ctx* ctx) {
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    if (ctx->d_model) (void)hipFree(ctx->d_model);
    if (ctx->d_ws) (void)hipFree(ctx->d_ws);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    if (ctx->h_status) (void)hipHostFree(ctx->h_status);
    for (hipEvent_t e : ctx->ev) if (e) (void)hipEventDestroy(e);
    delete ctx;
}

static int launch_encode(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, uint32_t* sf, float* params,
                         float* bits, hipStream_t st) {
    const uint32_t P = (uint32_t)((uint64_t)n * H * W);
    const EncodeVariant ev = kEncodeVariants[ctx->encode_variant];
    const uint32_t per_block = 16u * ev.tiles * (ev.threads / 64);
    uint32_t blocks = (P + per_block - 1) / per_block;
    const uint32_t cus = ctx->num_cus > 0 ? (uint32_t)ctx->num_cus : 256u;
    if (blocks > cus) blocks = cus;   // persistent: one workgroup per CU, looping over pixel groups
    switch (ctx->encode_variant) {
        case 0:
            hipLaunchKernelGGL((encode_kernel<1, 512>), dim3(blocks), dim3(512), kModelBytes, st, ctx->d_model, d_img,
                               H, W, P, sf, params, bits, ctx->d_status);
            break;
        case 1:
            hipLaunchKernelGGL((encode_kernel<2, 512>), dim3(blocks), dim3(512), kModelBytes, st, ctx->d_model, d_img,
                               H, W, P, sf, params, bits, ctx->d_status);
            break;
        default:
            hipLaunchKernelGGL((encode_kernel<1, 1024>), dim3(blocks), dim3(1024), kModelBytes, st, ctx->d_model, d_img,
                               H, W, P, sf, params, bits, ctx->d_status);
            break;
    }
    return hipGetLastError() == hipSuccess ? PCC_OK : PCC_E_HIP;
}

int pcc_encode_probs(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, float* d_params, float* d_bits,
                     void* hip_stream) {
    if (!ctx || !d_img || !d_params || !dims_ok(n, H, W)) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    return launch_encode(ctx, d_img, n, H, W, nullptr, d_params, d_bits, (hipStream_t)hip_stream);
}

int pcc_encode(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, uint8_t* d_stream, size_t cap_bytes,
               size_t* h_nbytes_out, void* hip_stream) {
    if (!ctx || !d_img || !d_stream || !h_nbytes_out || !dims_ok(n, H, W)) return PCC_E_ARG;
    if (((uintptr_t)d_stream & 7u) != 0) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    const uint64_t P = (uint64_t)n * H * W;
    const uint32_t rows = (uint32_t)((uint64_t)n * H);
    const size_t table = (size_t)kStreamHeader + 8 * ((size_t)rows + 1);
    if (cap_bytes < table) return PCC_E_CAP;

    const size_t sf_bytes = align_up(P * 3 * sizeof(uint32_t), 256);
    const size_t slab_bytes = align_up((size_t)rows * slab_words(W) * 4, 256);
    const size_t rw_bytes = align_up((size_t)rows * 4, 256);
    int rc = ensure_workspace(ctx, sf_bytes + slab_bytes + rw_bytes);
    if (rc != PCC_OK) return rc;
    uint32_t* d_sf = reinterpret_cast<uint32_t*>(ctx->d_ws);
    uint32_t* d_slabs = reinterpret_cast<uint32_t*>(ctx->d_ws + sf_bytes);
    uint32_t* d_rw = reinterpret_cast<uint32_t*>(ctx->d_ws + sf_bytes + slab_bytes);
    ctx->d_sf = d_sf;
    ctx->sf_count = (size_t)P * 3;

    if (hipMemsetAsync(ctx->d_status, 0, kStWords * sizeof(int) + sizeof(uint64_t), st) != hipSuccess) return PCC_E_HIP;
    prof_reset(ctx);
    prof_begin(ctx, PCC_T_ENCODE_PIXELS, st);
    rc = launch_encode(ctx, d_img, n, H, W, d_sf, nullptr, nullptr, st);
    if (rc != PCC_OK) return rc;
    prof_end(ctx, PCC_T_ENCODE_PIXELS, st);
    prof_begin(ctx, PCC_T_ENCODE_RANS, st);
    hipLaunchKernelGGL(rans_rows_kernel, dim3((rows + kRansRows - 1) / kRansRows), dim3(kRansRows), 0, st, d_sf, W, rows,
                       d_slabs, d_rw);
    prof_end(ctx, PCC_T_ENCODE_RANS, st);
    prof_begin(ctx, PCC_T_ENCODE_SCAN, st);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, d_rw, rows, n, H, W, ctx->dist, d_stream, ctx->d_total);
    prof_end(ctx, PCC_T_ENCODE_SCAN, st);
    prof_begin(ctx, PCC_T_ENCODE_COMPACT, st);
    hipLaunchKernelGGL(compact_kernel, dim3(rows), dim3(64), 0, st, d_slabs, d_rw, W, rows, d_stream,
                       (uint64_t)cap_bytes, ctx->d_status);
    prof_end(ctx, PCC_T_ENCODE_COMPACT, st);
    if (hipGetLastError() != hipSuccess) return PCC_E_HIP;
    if (hipMemcpyAsync(ctx->h_status, ctx->d_status, kStWords * sizeof(int) + sizeof(uint64_t), hipMemcpyDeviceToHost,
                       st) != hipSuccess) return PCC_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    prof_collect(ctx);
    if (ctx->h_status[kStErr] != 0) return ctx->h_status[kStErr];
    uint64_t total;
    memcpy(&total, ctx->h_status + kStWords, sizeof(total));
    if (total > cap_bytes) return PCC_E_CAP;
    *h_nbytes_out = (size_t)total;
    return PCC_OK;
}

int pcc_decode(pcc_ctx* ctx, const uint8_t* d_stream, size_t nbytes, int n, int H, int W, uint8_t* d_img_out,
               void* hip_stream) {
    if (!ctx || !d_stream || !d_img_out || !dims_ok(n, H, W)) return PCC_E_ARG;
    if (((uintptr_t)d_stream & 7u) != 0) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    hipStream_t st = (hipStream_t)hip_stream;
    const uint64_t rows = (uint64_t)n * H;
    const uint64_t table = (uint64_t)kStreamHeader + 8 * (rows + 1);
    if (nbytes < table + 8 * rows) return PCC_E_STREAM;   // every row payload holds at least its 8-byte state
    const int nbands = (H + kBandRows - 1) / kBandRows;
    const size_t mail_bytes = align_up((size_t)n * nbands * 2 * (size_t)W * 4, 256);
    int rc = ensure_workspace(ctx, mail_bytes);
    if (rc != PCC_OK) return rc;
    ctx->d_sf = nullptr; ctx->sf_count = 0;
    uint32_t* d_mail = reinterpret_cast<uint32_t*>(ctx->d_ws);
    if (hipMemsetAsync(ctx->d_status, 0, kStWords * sizeof(int) + sizeof(uint64_t), st) != hipSuccess) return PCC_E_HIP;
    if (hipMemsetAsync(d_mail, 0, mail_bytes, st) != hipSuccess) return PCC_E_HIP;
    const uint32_t spin_limit = 1u << 22;
    prof_reset(ctx);
    prof_begin(ctx, PCC_T_DECODE, st);
    const uint32_t grid = (uint32_t)(n * nbands);
    const uint32_t cus = ctx->num_cus > 0 ? (uint32_t)ctx->num_cus : 256u;
    if (grid <= cus)
        hipLaunchKernelGGL(decode_kernel<1>, dim3(grid), dim3(kDecThreads), kDecLdsBytes, st, ctx->d_model, d_stream,
                           (uint64_t)nbytes, n, H, W, nbands, ctx->dist, d_img_out, d_mail, ctx->d_status, spin_limit);
    else
        hipLaunchKernelGGL(decode_kernel<2>, dim3(grid), dim3(kDecThreads), kDecLdsBytes, st, ctx->d_model, d_stream,
                           (uint64_t)nbytes, n, H, W, nbands, ctx->dist, d_img_out, d_mail, ctx->d_status, spin_limit);
    prof_end(ctx, PCC_T_DECODE, st);
    if (hipGetLastError() != hipSuccess) return PCC_E_HIP;
    if (hipMemcpyAsync(ctx->h_status, ctx->d_status, kStWords * sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess)
        return PCC_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    prof_collect(ctx);
    return ctx->h_status[kStErr];
}

int pcc_cdf_tables(pcc_ctx* ctx, const float* d_params, const uint8_t* d_rg, size_t count, uint32_t* d_cq,
                   void* hip_stream) {
    if (!ctx || !d_params || !d_rg || !d_cq || count == 0 || count > (1u << 26)) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    const size_t threads = count * 3;
    hipLaunchKernelGGL(cdf_tables_kernel, dim3((uint32_t)((threads + 255) / 256)), dim3(256), (kLutEntries + 1) * 8,
                       (hipStream_t)hip_stream, ctx->d_model, d_params, d_rg, count, d_cq);
    return hipGetLastError() == hipSuccess ? PCC_OK : PCC_E_HIP;
}

int pcc_set_profiling(pcc_ctx* ctx, int enabled) {
    if (!ctx) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    if (enabled && !ctx->ev[0]) {
        for (hipEvent_t& e : ctx->ev)
            if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    }
    ctx->profiling = enabled != 0;
    prof_reset(ctx);
    return PCC_OK;
}

int pcc_last_timings(pcc_ctx* ctx, float* h_ms) {
    if (!ctx || !h_ms) return PCC_E_ARG;
    for (int i = 0; i < PCC_N_TIMINGS; ++i) h_ms[i] = ctx->last_ms[i];
    return PCC_OK;
}

#ifdef PCC_PHASE_TIMING
int pcc_debug_phase_cycles(unsigned long long* h_out16) {
    return hipMemcpyFromSymbol(h_out16, HIP_SYMBOL(pcc::g_phase_cycles), 16 * sizeof(unsigned long long)) == hipSuccess
               ? PCC_OK : PCC_E_HIP;
}
#endif

int pcc_copy_intervals(pcc_ctx* ctx, uint32_t* d_out, size_t count, void* hip_stream) {
    if (!ctx || !d_out) return PCC_E_ARG;
    if (!ctx->d_sf || count != ctx->sf_count) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    if (hipMemcpyAsync(d_out, ctx->d_sf, count * sizeof(uint32_t), hipMemcpyDeviceToDevice, (hipStream_t)hip_stream) !=
        hipSuccess) return PCC_E_HIP;
    return PCC_OK;
}

}  // extern "C"
