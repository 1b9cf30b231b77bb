// libpcc: kernels and C ABI (see include/pcc.h for the contract).
//
// Kernels (templated on the network description, see pcc_device.h)
//   encode_kernel      gather + network (MFMA) + mixture -> (start,freq) of the
//                      true sub-pixels, all pixels in parallel, the rows' right
//                      ends first
//   rans_rows_kernel   one lane per image row: push the row's symbols last to
//                      first into a per-row slab, written backwards; for a small
//                      job it runs beside encode_kernel, taking the symbols as
//                      they appear
//   scan_kernel        exclusive prefix sum of row payload sizes, header, offsets
//   compact_kernel     slabs -> contiguous stream
//   compact_scan_kernel  both of the above in one launch, for jobs of few rows
//   decode_kernel      persistent wavefront decoder: one workgroup (4 waves) per
//                      band of 16 rows, step t handles pixel (r, t - delay*r) of each row
//   cdf_tables_kernel  test hook: full integer CDF tables from given parameters
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "pcc.h"
#include "pcc_device.h"
#include "rans_arith.h"

namespace pcc {

constexpr uint32_t kBlobMagic = 0x57434350u;    // "PCCW"
constexpr uint32_t kStreamMagic = 0x31434350u;  // "PCC1"
constexpr int kStreamHeader = 32;
constexpr uint32_t kStreamVersion = 2;          // two coder states per row (1: one)
constexpr int kBandRows = 16;
constexpr uint32_t kMailTag = 0x80000000u;

template <class Net>
constexpr uint32_t model_tag() { return (uint32_t)Net::K | ((uint32_t)Net::kNbhd << 8) | ((uint32_t)Net::kDelay << 16) | (16u << 24); }

// Encode kernel variants: tiles of 16 pixels per wave per iteration x threads per workgroup.
// More tiles per wave reuse each LDS weight read more often but need more registers.
struct EncodeVariant { int tiles, threads; };
// pcc_encode_probs: pixels of a tile whose head outputs a wave stages in LDS at a time (four, or as many as fit
// beside the model image: two or one for the largest networks), and the bytes that takes for the workgroup.
constexpr int kLdsBytes = 160 * 1024;
// What the pixel kernel keeps in LDS: the weight tiles of as many leading layers as fit together with all biases,
// the biases behind them, and behind those the CDF table if there is room left (the whole model image when
// everything fits).  The other layers' tiles, and the table when it is not there, are read from global memory.
template <class Net>
constexpr int encode_resident_layers() {
    int r = Net::kLayers;
    while (r > 0 && Layout<Net>::w_off(r) + (Layout<Net>::kLutOff - Layout<Net>::kWeightBytes) > kLdsBytes) --r;
    return r;
}
template <class Net>
constexpr int encode_table_lds_off() {      // = Layout::kLutOff when all layers are resident
    return Layout<Net>::w_off(encode_resident_layers<Net>()) + (Layout<Net>::kLutOff - Layout<Net>::kWeightBytes);
}
template <class Net>
constexpr bool encode_table_in_lds() { return encode_table_lds_off<Net>() + (Layout<Net>::kModelBytes - Layout<Net>::kLutOff) <= kLdsBytes; }
template <class Net>
constexpr int encode_model_lds_bytes() {
    return encode_table_lds_off<Net>() + (encode_table_in_lds<Net>() ? Layout<Net>::kModelBytes - Layout<Net>::kLutOff : 0);
}
// 0: no room for a staging area; the head outputs are then stored value by value.
template <class Net>
constexpr int params_stage_pixels(int threads) {
    for (int px = 4; px >= 1; px /= 2)
        if (encode_model_lds_bytes<Net>() + (threads / 64) * px * Net::dim(Net::kLayers) * 4 <= kLdsBytes) return px;
    return 0;
}
template <class Net>
constexpr int params_stage_bytes(int threads) { return (threads / 64) * params_stage_pixels<Net>(threads) * Net::dim(Net::kLayers) * 4; }
constexpr EncodeVariant kEncodeVariants[4] = {{1, 512}, {2, 512}, {1, 1024}, {4, 256}};

// status words in device memory
enum { kStErr = 0, kStAbort = 1, kStTicket = 2, kStWords = 4 };
// The status block: kStWords ints that every call clears on its stream before its kernels, the 64-bit stream
// size, and two ints that only a row coder running beside the pixel kernel writes (stood down; spare).
// That row coder runs on another stream than the clearing, so its words are cleared after they have been read,
// at the end of the call, and are zero whenever a call begins.
constexpr size_t kStCleared = kStWords * sizeof(int) + sizeof(uint64_t);
constexpr int kStSide = (int)(kStCleared / sizeof(int));     // index of the first of the two side words
enum { kSideDefer = 0 };
constexpr size_t kStBytes = kStCleared + 2 * sizeof(int);

// Most 32-bit words a row's payload can have: four of the two final coder states, and one per two symbols plus two.
__host__ __device__ inline size_t slab_words(int W) { return (6 * (size_t)W + 24) / 4 + 1; }

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

__device__ __forceinline__ void copy_to_lds(uint8_t* lds, const uint8_t* __restrict__ src, int bytes) {
    const uint4* s = reinterpret_cast<const uint4*>(src);
    uint4* d = reinterpret_cast<uint4*>(lds);
    for (int i = threadIdx.x; i < bytes / 16; i += blockDim.x) d[i] = s[i];
}

// Lane group and register (g * kHeadSlots + s) that hold canonical head output c.
template <class Net>
__host__ __device__ constexpr int head_slot(int c) {
    for (int g = 0; g < 4; ++g)
        for (int s = 0; s < Layout<Net>::kHeadSlots; ++s)
            if (Net::head_index(g, s) == c) return g * Layout<Net>::kHeadSlots + s;
    return -1;
}

// Compile-time loop: f(std::integral_constant<int, I>) for I = 0 .. N-1.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Raw head registers of one lane after the network -> mixture of "its" channel
// (lane groups 0,1,2 = R,G,B) with the coupling coefficients it needs.
template <class Net>
struct LaneHead {
    ChanParams<Net::K> cp;
    float c1[Net::K];  // alpha (group 1) or beta (group 2)
    float c2[Net::K];  // gamma (group 2)
};

template <class Net>
__device__ __forceinline__ void lane_head_setup(const f32x4_t (&o)[Layout<Net>::kHeadOB], int lane, float lut_scale,
                                                LaneHead<Net>& h) {
    constexpr int K = Net::K, HS = Layout<Net>::kHeadSlots;
    float v[HS];
#pragma unroll
    for (int ob = 0; ob < Layout<Net>::kHeadOB; ++ob) {
        v[4 * ob + 0] = o[ob].x; v[4 * ob + 1] = o[ob].y; v[4 * ob + 2] = o[ob].z; v[4 * ob + 3] = o[ob].w;
    }
    const int g = lane >> 4, nl = lane & 15;
    float raw[3 * K];
#pragma unroll
    for (int s = 0; s < 3 * K; ++s) raw[s] = v[s];
    channel_setup<K>(raw, lut_scale, h.cp);
    // Coupling coefficients alpha_k = head[9K+k] (needed by group 1), beta_k = head[10K+k] and
    // gamma_k = head[11K+k] (group 2): the lane's own register where its group holds the value,
    // else pulled from the lane of the same pixel in the group that does.
    static_for<0, K>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        constexpr int sa = head_slot<Net>(9 * K + k), sb = head_slot<Net>(10 * K + k), sc = head_slot<Net>(11 * K + k);
        static_assert(sa >= 0 && sb >= 0 && sc >= 0, "every head output has a register");
        float va, vb, vc;
        if constexpr (sa / HS == 1) va = v[sa % HS]; else va = __shfl(v[sa % HS], nl + 16 * (sa / HS));
        if constexpr (sb / HS == 2) vb = v[sb % HS]; else vb = __shfl(v[sb % HS], nl + 16 * (sb / HS));
        if constexpr (sc / HS == 2) vc = v[sc % HS]; else vc = __shfl(v[sc % HS], nl + 16 * (sc / HS));
        h.c1[k] = (g == 1) ? va : vb;
        h.c2[k] = vc;
    });
}

// ---------------------------------------------------------------------------
// encode: all pixels in parallel
//
// A work item is a strip of 16 T consecutive pixels of one image row; strips are
// numbered from the right edge of the image, item = strip * rows + row, and wave
// w of the grid's G waves takes the items w, w + G, w + 2G, ...  The rows' right
// ends are therefore finished first, which is where the row coder starts (it
// pushes the symbols last to first).  The row coder may run beside this kernel:
// then the results go to sf_tagged instead of sf, one 64-bit word per symbol with
// this launch's epoch in the high half, written through to device scope.  A
// reader that finds the epoch has the symbol; nothing else is published and
// nothing has to be cleared between launches (epochs only grow).
// ---------------------------------------------------------------------------
template <class Net, int T, int THREADS>
__global__ void __launch_bounds__(THREADS)
encode_kernel(const uint8_t* __restrict__ model, const uint8_t* __restrict__ img, int n, int H, int W,
              uint32_t* __restrict__ sf, float* __restrict__ params, float* __restrict__ bits, int* status,
              uint64_t* sf_tagged, uint32_t epoch, uint32_t strip_begin, uint32_t strip_count) {
    using Lay = Layout<Net>;
    constexpr int K = Net::K, KB0 = Net::kb(0), HEAD = Net::dim(Net::kLayers);
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int RESIDENT = encode_resident_layers<Net>();
    if constexpr (RESIDENT == Net::kLayers) {
        copy_to_lds(lds, model, encode_model_lds_bytes<Net>());
    } else {
        copy_to_lds(lds, model, Lay::w_off(RESIDENT));
        copy_to_lds(lds + Lay::w_off(RESIDENT), model + Lay::kWeightBytes, encode_model_lds_bytes<Net>() - Lay::w_off(RESIDENT));
    }
    __syncthreads();
    const uint8_t* table_at = encode_table_in_lds<Net>() ? lds + (encode_table_lds_off<Net>() - Lay::kLutOff) : model;
    const float2* lut = reinterpret_cast<const float2*>(table_at + Lay::kLutOff);
    const float lut_scale = *reinterpret_cast<const float*>(table_at + Lay::kLutScaleOff);
    const int lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // a scalar: the item's row and strip are scalars too
    const int g = lane >> 4, nl = lane & 15;
    const uint32_t rows = (uint32_t)n * (uint32_t)H;
    const uint32_t P = rows * (uint32_t)W;
    const uint32_t items = strip_count * rows;              // this launch's strips: strip_begin .. strip_begin + strip_count - 1
    for (uint32_t item = blockIdx.x * nwaves + wave; item < items; item += gridDim.x * nwaves) {
        const uint32_t local = item / rows, rowg = item - local * rows, strip = strip_begin + local;
        const uint32_t im = rowg / (uint32_t)H;
        const int r = (int)(rowg - im * (uint32_t)H);
        const int c0 = W - 16 * T * (int)(strip + 1);           // negative in the leftmost strip of a ragged width
        const uint8_t* base = img + (size_t)im * H * W * 3;
        u32x4_t in[T][KB0][2];
        uint32_t pix[T];   // the pixel's own bytes r | g<<8 | b<<16
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int c = c0 + 16 * t + nl;
            uint32_t runs[KB0][2];
#pragma unroll
            for (int kbi = 0; kbi < KB0; ++kbi) { runs[kbi][0] = 0; runs[kbi][1] = 0; }
            pix[t] = 0;
            if (c >= 0) {
                const uint32_t p = rowg * (uint32_t)W + (uint32_t)c;
                const int me = (r * W + c) * 3;
                if (p + 1 < P) {
                    uint32_t v;
                    __builtin_memcpy(&v, base + me, 4);       // unaligned dword; the fourth byte is the next pixel's
                    pix[t] = v & 0xFFFFFFu;
                } else {
                    pix[t] = (uint32_t)base[me] | ((uint32_t)base[me + 1] << 8) | ((uint32_t)base[me + 2] << 16);
                }
                // This lane's first-layer inputs are runs of four consecutive image bytes; a run is
                // read with one load when all its bytes lie in the image, byte by byte at the borders.
#pragma unroll
                for (int kbi = 0; kbi < KB0; ++kbi) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        int dr = 0, off = 0;
                        if (!Net::run_desc(kbi, g, half, dr, off)) continue;
                        const int rr = r + dr;
                        const int at = (rr * W + (c - 2)) * 3 + off;
                        const int col_first = c - 2 + ((off * 11) >> 5), col_last = c - 2 + (((off + 3) * 11) >> 5);
                        uint32_t v = 0;
                        if (rr >= 0 && col_first >= 0 && col_last < W) {
                            __builtin_memcpy(&v, base + at, 4);
                        } else if (rr >= 0) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int col = c - 2 + (((off + i) * 11) >> 5);
                                if (col >= 0 && col < W) v |= (uint32_t)base[at + i] << (8 * i);
                            }
                        }
                        runs[kbi][half] = v;
                    }
                }
            }
#pragma unroll
            for (int kbi = 0; kbi < KB0; ++kbi) {
                uint32_t a, b, c2, d;
                run_to_bf16(runs[kbi][0], a, b);
                run_to_bf16(runs[kbi][1], c2, d);
                in[t][kbi][0].x = a; in[t][kbi][0].y = b; in[t][kbi][0].z = c2; in[t][kbi][0].w = d;
                in[t][kbi][1] = in[t][kbi][0];   // unused (layer-1 inputs are exact)
            }
        }
        f32x4_t out[T][Lay::kHeadOB];
        mlp_from<Net, T, (T == 1 && THREADS <= 512), 0, RESIDENT>(lds + opaque_zero(), model, lane, in, out);
        // The head's results are first read behind branches (which outputs are wanted, border tiles).  The wait
        // states an MFMA's result needs are counted along the instruction stream as laid out, not along a taken
        // branch, so the accumulators are made to settle here, in straight-line code.
#pragma unroll
        for (int t = 0; t < T; ++t) {
#pragma unroll
            for (int ob = 0; ob < Lay::kHeadOB; ++ob) asm volatile("" : "+v"(out[t][ob]));
        }
        asm volatile("s_nop 7" ::: "memory");

#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int c = c0 + 16 * t + nl;
            const bool live = c >= 0;
            const uint32_t p = rowg * (uint32_t)W + (uint32_t)c;
            constexpr int kStagePixels = params_stage_pixels<Net>(THREADS);
            constexpr int PX = kStagePixels > 0 ? kStagePixels : 1;       // (the block below is dead code when there is no room)
            if (kStagePixels > 0 && params != nullptr && ((uintptr_t)params & 15u) == 0) {
                // The tile's head outputs are HEAD consecutive floats per pixel, 16 consecutive pixels: they go
                // through a staging area of this wave in LDS, PX pixels at a time, and leave as
                // 16-byte stores of consecutive lanes (stored straight from the registers, a lane's values lie
                // 4 bytes here and 4 bytes there, 240 bytes apart from its neighbour's).  LDS takes a wave's
                // instructions in order, so the reads see the writes of the same pass.
                float* stage = reinterpret_cast<float*>(lds + encode_model_lds_bytes<Net>()) + wave * (PX * HEAD);
#pragma unroll
                for (int pass = 0; pass < 16 / PX; ++pass) {
                    if (nl / PX == pass) {
#pragma unroll
                        for (int ob = 0; ob < Lay::kHeadOB; ++ob) {
                            const float vv[4] = {out[t][ob].x, out[t][ob].y, out[t][ob].z, out[t][ob].w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int idx = Net::head_index(g, 4 * ob + i);
                                if (idx >= 0) stage[(nl % PX) * HEAD + idx] = vv[i];
                            }
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                    for (int j = lane; j < PX * HEAD / 4; j += 64) {
                        const int cc = c0 + 16 * t + pass * PX + (4 * j) / HEAD;      // the chunk's pixel
                        if (cc >= 0) {
                            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(stage + 4 * j);
                            *reinterpret_cast<f32x4_t*>(params + ((size_t)rowg * W + cc) * HEAD + (4 * j) % HEAD) = v;
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            } else if (params != nullptr && live) {
#pragma unroll
                for (int ob = 0; ob < Lay::kHeadOB; ++ob) {
                    const float vv[4] = {out[t][ob].x, out[t][ob].y, out[t][ob].z, out[t][ob].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int idx = Net::head_index(g, 4 * ob + i);
                        if (idx >= 0) params[(size_t)p * HEAD + idx] = vv[i];
                    }
                }
            }
            LaneHead<Net> h;
            lane_head_setup<Net>(out[t], lane, lut_scale, h);
            const float rhat = (float)(pix[t] & 0xFF) * (1.0f / 256.0f);
            const float ghat = (float)((pix[t] >> 8) & 0xFF) * (1.0f / 256.0f);
            if (g == 1) couple_green<K>(h.cp, h.c1, rhat);
            if (g == 2) couple_blue<K>(h.cp, h.c1, h.c2, rhat, ghat);
            const int x = (int)((pix[t] >> (8 * (g & 3))) & 0xFF);   // group 3 reads the zero top byte
            const uint32_t lo = cq_full<K>(h.cp, x, lut);
            const uint32_t hi = cq_full<K>(h.cp, x + 1, lut);
            uint32_t freq = hi - lo;
            if (g < 3 && live && (hi <= lo || freq > 65536u)) { set_error(status, PCC_E_INTERNAL); freq = 1; }
            if (g < 3 && live) {
                const uint32_t word = lo | ((freq - 1u) << 16);
                if (sf_tagged != nullptr)
                    __hip_atomic_store(&sf_tagged[(size_t)p * 3 + g], ((uint64_t)epoch << 32) | word, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                else if (sf != nullptr) sf[(size_t)p * 3 + g] = word;
            }
            if (bits != nullptr) {
                const float mine = 16.0f - __builtin_amdgcn_logf((float)freq);
                const float tot = (__shfl(mine, nl) + __shfl(mine, nl + 16)) + __shfl(mine, nl + 32);
                if (g == 0 && live) bits[p] = tot;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// rANS encode, two lanes per row: one per coder state.  A row's stream carries
// two interleaved states (symbol i on state i mod 2) that meet only in the order
// of the words they emit, so each state's serial chain runs in a lane of its
// own and the order is restored afterwards.  A workgroup owns 32 rows: the 64
// lanes of wave 0 each run one state's chain; waves 2 and 3 fetch the rows'
// (start, freq) words chunk by chunk (coalesced, two chunks ahead), compute the
// fp64 reciprocal of every frequency and stage both in LDS; wave 1 merges the
// words the two lanes of a row produced, in the order of the symbols that
// caused them, and copies them from LDS to the rows' slabs.  The coding wave's
// instruction stream, which bounds the kernel (it is limited by instruction
// issue, not by the latency of the chain), then holds only the chain itself.
// ---------------------------------------------------------------------------
constexpr int kRansRows = 32;
constexpr int kRansChunk = 64;                      // symbols of a row per round: 32 for each of its two lanes
constexpr int kRansThreads = 256;
constexpr uint32_t kRansBesideMaxGroups = 96;      // row-coder workgroups that may run beside the pixel kernel
constexpr uint32_t kXcds = 8;
constexpr uint32_t kRansPatience = 2048;            // polls for one symbol before a row coder beside the pixel kernel stands down (a few ms)
// Rows at which the row coder of an image takes as long as the pixel kernel with the whole chip (both times are
// proportional to the width; measured with the 30-160-160-128-60 network, 768x512 to 4096x2160): decides how much of
// a tall image the pixel kernel does before the row coder joins it.
constexpr uint32_t kRansBalanceRows = 600;
// Padding symbol (start 0, frequency 2^16): pushing it leaves the state unchanged
// and never renormalises, so every chunk can be coded as a full one.
constexpr uint32_t kRansNop = 0xFFFF0000u;

// The coding wave rounds its fp64 arithmetic toward zero (MODE.FP_ROUND bits 3:2 = 3).  Written as
// assembly: the compiler would put the default mode back in front of the wave's fp64 instructions.
// rans_push (rans_arith.h) relies on it.
__device__ __forceinline__ void rans_round_toward_zero() {
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 3" ::: "memory");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for
// every outstanding global access (stores, polls, prefetches), which would put
// memory latency on the critical path of every round of the row coder and several
// times on every step of the decoder; neither hands global data from thread to
// thread across such a barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// BESIDE: the pixel kernel is running; the symbols are read from sf_tagged, past the caches that are not
// coherent with the pixel kernel's stores, and each is waited for until it carries this launch's epoch.
template <bool BESIDE>
__global__ void __launch_bounds__(kRansThreads)
rans_rows_kernel(const uint32_t* __restrict__ sf, const uint64_t* sf_tagged, uint32_t epoch, int W, uint32_t rows,
                 uint32_t* __restrict__ slabs, uint32_t* __restrict__ row_words, int* status, uint32_t patience) {
    constexpr int kPerState = kRansChunk / 2;   // symbols of a chunk that one state (one coding lane) takes
    static_assert(kPerState == 32, "a coding lane's emission flags of a round fill one 32-bit word");
    // [buffer][row][symbol of the chunk]; the odd row strides keep the coding wave's column accesses off shared banks
    __shared__ uint32_t sym[2][kRansRows][kRansChunk + 1];
    __shared__ double rcp[2][kRansRows][kRansChunk + 1];
    // [buffer][state][row][step]: the low state word before each of the lane's symbols of the chunk, in the order
    // coded; it is one of the stream's words where the lane's flag for that step is set
    __shared__ uint32_t outw[2][2][kRansRows][kPerState + 1];
    // [buffer][row][state]: the flags, the first step's in bit 31
    __shared__ uint32_t outflags[2][kRansRows][2];
    __shared__ uint32_t final_state[kRansRows][4];   // xl, xh of state 0, xl, xh of state 1 after the row's first symbol
    __shared__ uint32_t abandon;                // set by a loader whose wait ran out: every wave leaves after the round
    const int tid = threadIdx.x, lane = tid & 63;
    const bool coder = tid < 64;
    const uint32_t row0 = blockIdx.x * kRansRows;
    const uint32_t nsym = 3u * (uint32_t)W;
    const int nchunks = (int)((nsym + kRansChunk - 1) / kRansChunk);
    const uint32_t live_rows = min((uint32_t)kRansRows, rows - row0);
    const size_t sw = slab_words(W);
    // coding lane: row of the workgroup lane & 31, state lane >> 5 (symbol i of the row is coded on state i mod 2)
    const int crow = lane & (kRansRows - 1), cstate = lane >> 5;
    uint32_t xl = (uint32_t)kRansL, xh = (uint32_t)(kRansL >> 32);     // the lane's state x = xh 2^32 + xl
    // storing lanes keep the slab position of row lane & 31: slabs fill from the end, the decoder reads the words in
    // reverse order of production
    uint32_t wp = (uint32_t)sw;

    // Wave 0 codes; waves 2 and 3 load (symbols from global memory, reciprocals, both to LDS); wave 1 stores (the
    // words the coding wave produced, from LDS to the rows' slabs).  Loads and stores are kept in different waves
    // because a wave's loads and stores complete out of order with each other under one counter: a wave that
    // has stores in flight can only wait for a load by waiting for everything.
    const bool storer = tid >= 64 && tid < 128, loader = tid >= 128;
    constexpr int kLoaders = kRansThreads - 128;
    constexpr int kPerLoader = (kRansRows * kRansChunk + kLoaders - 1) / kLoaders;
    static_assert(kRansRows * kRansChunk % kLoaders == 0 && kRansRows == 32, "whole elements per thread; a row per lane pair");
    static_assert(kRansChunk % 2 == 0, "a chunk starts at an even symbol index: the state of a symbol follows from its place in the chunk");
    // The pipeline, one stage per round (a round = the coding wave codes a chunk; rounds end in a workgroup
    // barrier), so that no wave waits for memory inside a round:
    //   round k + 3  the chunk's symbols are requested from global memory into registers (two sets, by round parity)
    //   round k + 1  (beside the pixel kernel: symbols it has not written yet are waited for,) reciprocals are
    //                computed, symbols and reciprocals go to LDS buffer k & 1
    //   round k      the coding wave codes the chunk
    //   round k - 1  the words it produced are copied to the rows' slabs
    using Staged = std::conditional_t<BESIDE, uint64_t, uint32_t>;
    Staged staged[2][kPerLoader];
    auto request = [&](int k, Staged (&staged)[kPerLoader]) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < kPerLoader; ++it) {
            const int e = tid - 128 + it * kLoaders;
            const uint32_t r = (uint32_t)e / kRansChunk, i = (uint32_t)e % kRansChunk;
            const uint32_t idx = (uint32_t)k * kRansChunk + i;
            // every lane loads (a padding element loads the buffer's first word): with no branch round the loads
            // the compiler can count them, and waits for one register set while the other's loads are in flight
            const bool real = r < live_rows && idx < nsym;
            const size_t at = real ? (size_t)(row0 + r) * nsym + idx : 0;
            if constexpr (BESIDE) staged[it] = __hip_atomic_load(&sf_tagged[at], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else staged[it] = sf[at];
        }
    };
    auto deposit = [&](int k, Staged (&staged)[kPerLoader]) __attribute__((always_inline)) {
        const int b = k & 1;
        if constexpr (BESIDE) {
            // Symbols the pixel kernel has not written yet (seldom once the pixel kernel, the faster of the two, is
            // ahead): the lane polls one of them, sleeping in between so that the polls of a coder that has
            // caught up do not load the memory system, and then loads its whole set again, all loads at once.
            // A running pixel kernel delivers a row's next strip within tens of microseconds.  A wait of
            // `patience` polls (milliseconds) therefore means that it is not running beside this kernel
            // (something runs the process's kernels one at a time, or the chip is taken): the row coder stands
            // down, and the host launches it again after the pixel kernel.
            uint32_t spins = 0;
            for (;;) {
                size_t stale_at = 0;
                bool stale = false;
#pragma unroll
                for (int it = 0; it < kPerLoader; ++it) {
                    const int e = tid - 128 + it * kLoaders;
                    const uint32_t r = (uint32_t)e / kRansChunk, i = (uint32_t)e % kRansChunk;
                    const uint32_t idx = (uint32_t)k * kRansChunk + i;
                    if (r < live_rows && idx < nsym && (uint32_t)(staged[it] >> 32) != epoch) {
                        stale = true;
                        stale_at = (size_t)(row0 + r) * nsym + idx;
                    }
                }
                if (!stale) break;
                bool gave_up = false;
                while ((uint32_t)(__hip_atomic_load(&sf_tagged[stale_at], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32) != epoch) {
                    if (++spins > patience) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(32);
                }
                if (gave_up) {
                    __hip_atomic_store(&status[kStSide + kSideDefer], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    abandon = 1;
                    break;
                }
                request(k, staged);
            }
        }
#pragma unroll
        for (int it = 0; it < kPerLoader; ++it) {
            const int e = tid - 128 + it * kLoaders;
            const uint32_t r = (uint32_t)e / kRansChunk, i = (uint32_t)e % kRansChunk;
            const bool real = r < live_rows && (uint32_t)k * kRansChunk + i < nsym;
            const uint32_t v = real ? (uint32_t)staged[it] : kRansNop;
            sym[b][r][i] = v;
            rcp[b][r][i] = rans_recip_below((v >> 16) + 1u);
        }
    };
    // Wave 1: the words of a finished chunk from buffer b to the rows' slabs, one row per iteration.  Lane p stands
    // for the p-th symbol coded in the round (symbol kRansChunk - 1 - p of the chunk: state 1 when p is even, the
    // state's step p / 2).  Where that symbol's flag is set, its word goes behind the words of the symbols coded
    // before it, from either state: the flags set among the first ceil(p / 2) steps of state 1 and the first
    // floor(p / 2) steps of state 0.  All LDS reads are issued before the first store.
    auto flush = [&](int b) __attribute__((always_inline)) {
        const uint32_t p = (uint32_t)lane, step = p >> 1, state = 1u - (p & 1u);
        auto first_steps = [](uint32_t nsteps) { return nsteps == 0 ? 0u : 0xFFFFFFFFu << (32u - nsteps); };   // their flag bits
        const uint32_t before1 = first_steps((p + 1) >> 1), before0 = first_steps(p >> 1), mine = 0x80000000u >> step;
        uint32_t word[kRansRows], f0[kRansRows], f1[kRansRows];
#pragma unroll
        for (int r = 0; r < kRansRows; ++r) {
            word[r] = outw[b][state][r][step];
            f0[r] = outflags[b][r][0];
            f1[r] = outflags[b][r][1];
        }
        const uint32_t own0 = outflags[b][lane & (kRansRows - 1)][0], own1 = outflags[b][lane & (kRansRows - 1)][1];
#pragma unroll
        for (int r = 0; r < kRansRows; ++r) {
            const uint32_t at = (uint32_t)__builtin_amdgcn_readlane((int)wp, r);     // the row's position before this chunk
            const uint32_t ahead = (uint32_t)__popc(f1[r] & before1) + (uint32_t)__popc(f0[r] & before0);
            const bool emitted = ((state ? f1[r] : f0[r]) & mine) != 0;
            if ((uint32_t)r < live_rows && emitted) slabs[(size_t)(row0 + r) * sw + (at - 1u - ahead)] = word[r];
        }
        wp -= (uint32_t)__popc(own0) + (uint32_t)__popc(own1);
    };
    if (tid == 0) abandon = 0;
    lds_barrier();
    if (coder) rans_round_toward_zero();
    // one round; P = the round's parity, which picks the loaders' register set
    auto round = [&](int k, auto parity) __attribute__((always_inline)) {
        constexpr int P = decltype(parity)::value;
        const int b = k & 1;
        if (loader) {
            if (k >= 1 && k - 1 < nchunks) deposit(k - 1, staged[P]);
            request(min(max(k - 3, 0), nchunks - 1), staged[P]);     // outside the chunks: loads nobody uses
        } else if (storer) {
            if (k >= -1 && k + 1 < nchunks) flush(b ^ 1);
        } else if (k >= 0 && k < nchunks) {
            // The lane's symbols of the chunk, last first: kRansChunk - 2 + cstate, then every second one down to
            // cstate.  Symbols and reciprocals come from LDS in batches of kU; the next batch is requested before
            // the serial chain of the current one starts, so that only the round's first read waits for LDS.
            constexpr int kU = 8, kBatches = kPerState / kU;
            uint32_t v[2][kU];
            double rf[2][kU];
            const uint32_t* my_sym = &sym[b][crow][cstate];
            const double* my_rcp = &rcp[b][crow][cstate];
            uint32_t* my_out = &outw[b][cstate][crow][0];
            auto fetch = [&](int n) {
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    v[n & 1][u] = my_sym[kRansChunk - 2 - 2 * (n * kU + u)];
                    rf[n & 1][u] = my_rcp[kRansChunk - 2 - 2 * (n * kU + u)];
                }
            };
            uint32_t flags = 0;
            fetch(0);
#pragma unroll
            for (int n = 0; n < kBatches; ++n) {
                if (n + 1 < kBatches) fetch(n + 1);
#pragma unroll
                for (int u = 0; u < kU; ++u) {
                    const uint32_t start = v[n & 1][u] & 0xFFFFu, f = (v[n & 1][u] >> 16) + 1u;
                    // renormalise when x >= f * 2^47; the low word is stored either way, at the step's own place,
                    // and only counts where the flag says it was due: no branch and no address arithmetic on the
                    // serial chain
                    const bool emit = (xh >> 15) >= f;
                    my_out[n * kU + u] = xl;
                    flags = (flags << 1) | (emit ? 1u : 0u);
                    xl = emit ? xh : xl;
                    xh = emit ? 0u : xh;
                    rans_push(xl, xh, f, start, rf[n & 1][u]);
                }
            }
            outflags[b][crow][cstate] = flags;
        }
        lds_barrier();   // all that crosses threads here is in LDS; the loaders' global loads stay in flight
        return !BESIDE || abandon == 0;
    };
    // rounds nchunks + 2 (or + 3, for an even number of rounds) down to -1, where chunk 0's words are stored
    for (int k = nchunks + 2 + (nchunks & 1); k >= 0; k -= 2) {
        if (!round(k, std::integral_constant<int, 0>()) || !round(k - 1, std::integral_constant<int, 1>())) {
            if (tid < kRansRows && row0 + tid < rows) row_words[row0 + tid] = 0;    // stood down: nothing for the compaction to copy
            return;
        }
    }
    if (coder) {
        final_state[crow][2 * cstate] = xl;
        final_state[crow][2 * cstate + 1] = xh;
    }
    lds_barrier();
    if (storer && lane < kRansRows && row0 + lane < rows) {
        // the four state words end the slab's data: the decoder reads them first
        uint32_t* slab = slabs + (size_t)(row0 + lane) * sw;
        slab[wp - 1] = final_state[lane][3];
        slab[wp - 2] = final_state[lane][2];
        slab[wp - 3] = final_state[lane][1];
        slab[wp - 4] = final_state[lane][0];
        row_words[row0 + lane] = (uint32_t)sw - (wp - 4u);
    }
}

// Single workgroup: offsets[k] = 4 * sum_{j<k} row_words[j]; header; total size.
__global__ void __launch_bounds__(1024)
scan_kernel(const uint32_t* __restrict__ row_words, uint32_t rows, int n, int H, int W, uint32_t tag, uint32_t dist,
            uint8_t* __restrict__ stream, uint64_t* __restrict__ total_bytes) {
    __shared__ uint64_t part[1024];
    __shared__ uint64_t carry;
    uint64_t* offsets = reinterpret_cast<uint64_t*>(stream + kStreamHeader);
    if (threadIdx.x == 0) {
        carry = 0;
        uint32_t* hdr = reinterpret_cast<uint32_t*>(stream);
        hdr[0] = kStreamMagic; hdr[1] = kStreamVersion; hdr[2] = (uint32_t)n; hdr[3] = (uint32_t)H; hdr[4] = (uint32_t)W;
        hdr[5] = tag; hdr[6] = dist; hdr[7] = 0;
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
    if (nw > sw) {                                // not a row coder's count: never read outside the slab
        if (threadIdx.x == 0) set_error(status, PCC_E_INTERNAL);
        return;
    }
    if (table + off + 4ull * nw > cap_bytes) {
        if (threadIdx.x == 0) set_error(status, PCC_E_CAP);
        return;
    }
    const uint32_t* src = slabs + (size_t)row * sw + (sw - nw);
    uint32_t* dst = reinterpret_cast<uint32_t*>(stream + table + off);
    for (uint32_t i = threadIdx.x; i < nw; i += blockDim.x) dst[i] = src[i];
}

// test hook: the symbols of a tagged buffer without their epochs
__global__ void __launch_bounds__(256)
untag_kernel(const uint64_t* __restrict__ tagged, size_t count, uint32_t* __restrict__ out) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) out[i] = (uint32_t)tagged[i];
}

// scan_kernel and compact_kernel in one launch for jobs of few rows: every workgroup sums the sizes of the rows
// before its own (the sizes stay in L2), so nothing has to wait for a scan.  Quadratic in the rows.
constexpr uint32_t kCompactScanMaxRows = 4096;
constexpr int kCompactScanThreads = 256;

__global__ void __launch_bounds__(kCompactScanThreads)
compact_scan_kernel(const uint32_t* __restrict__ slabs, const uint32_t* __restrict__ row_words, int n, int H, int W,
                    uint32_t rows, uint32_t tag, uint32_t dist, uint8_t* __restrict__ stream, uint64_t cap_bytes,
                    uint64_t* __restrict__ total_bytes, int* status) {
    __shared__ unsigned long long part[kCompactScanThreads / 64];
    const uint32_t row = blockIdx.x;
    unsigned long long words_before = 0;
    for (uint32_t j = threadIdx.x; j < row; j += kCompactScanThreads) words_before += row_words[j];
    for (int d = 32; d >= 1; d >>= 1) words_before += __shfl_xor(words_before, d);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = words_before;
    __syncthreads();
    words_before = 0;
    for (int w = 0; w < kCompactScanThreads / 64; ++w) words_before += part[w];

    const size_t sw = slab_words(W);
    const uint64_t table = (uint64_t)kStreamHeader + 8ull * (rows + 1);
    const uint64_t off = 4ull * words_before;
    const uint32_t nw = row_words[row];
    // header, this row's offset and, from the last row, the end offset and the total: all inside the table,
    // which the host has checked against the capacity
    uint64_t* offsets = reinterpret_cast<uint64_t*>(stream + kStreamHeader);
    if (threadIdx.x == 0) {
        offsets[row] = off;
        if (row == 0) {
            uint32_t* hdr = reinterpret_cast<uint32_t*>(stream);
            hdr[0] = kStreamMagic; hdr[1] = kStreamVersion; hdr[2] = (uint32_t)n; hdr[3] = (uint32_t)H; hdr[4] = (uint32_t)W;
            hdr[5] = tag; hdr[6] = dist; hdr[7] = 0;
        }
        if (row + 1 == rows) {
            offsets[rows] = off + 4ull * nw;
            *total_bytes = table + off + 4ull * nw;
        }
    }
    if (nw > sw) {                                // not a row coder's count: never read outside the slab
        if (threadIdx.x == 0) set_error(status, PCC_E_INTERNAL);
        return;
    }
    if (table + off + 4ull * nw > cap_bytes) {
        if (threadIdx.x == 0) set_error(status, PCC_E_CAP);
        return;
    }
    const uint32_t* src = slabs + (size_t)row * sw + (sw - nw);
    uint32_t* dst = reinterpret_cast<uint32_t*>(stream + table + off);
    for (uint32_t i = threadIdx.x; i < nw; i += kCompactScanThreads) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// wavefront decode
//
// One workgroup of 4 waves owns a band of 16 image rows; step t decodes pixel
// (r, t - delay * r) of each row (delay = right reach of the neighbourhood + 1).
// Per step:
//   network   the 16 pixels form one MFMA tile; each wave computes a quarter
//             of every layer's out-blocks with its weight slices held in
//             registers for the whole kernel, and the layers meet in LDS
//   search    16 lanes per pixel find the symbol with two 16-way sweeps of
//             Cq evaluations per channel (R, then G given R, then B given R,G)
//   publish   the pixel goes to the LDS ring (next steps' neighbourhoods), to
//             the output image and, for the band's last two rows, to a mailbox
//             in global memory that the band below polls
// ---------------------------------------------------------------------------
constexpr int kDecThreads = 256;

// Where a decode step spends its cycles: built only with -DPCC_PHASE_TIMING (a measurement build; the product has
// an empty struct here and no code).  Every wave reads the shader clock at the marks of the step and sums the
// differences per phase; the workgroup that decodes ticket kPhaseTicket leaves the sums in phase_cycles.
enum { kPhGather = 0, kPhLayer0 = 1 /* + layer */, kPhMixture = 8, kPhR = 9, kPhG = 10, kPhB = 11, kPhPublish = 12,
       kPhFetch = 13, kPhBarrier = 14, kPhTop = 15, kPhCount = 16 };
#ifdef PCC_PHASE_TIMING
constexpr int kPhaseTicket = 8;
__device__ unsigned long long phase_cycles[4][kPhCount + 1];
struct PhaseClock {
    uint64_t t, acc[kPhCount];
    __device__ __forceinline__ void reset() {
        for (int i = 0; i < kPhCount; ++i) acc[i] = 0;
        t = __builtin_readcyclecounter();
    }
    __device__ __forceinline__ void mark(int i) {
        __builtin_amdgcn_sched_barrier(0);      // no instruction of one phase is moved into another
        const uint64_t now = __builtin_readcyclecounter();
        acc[i] += now - t;
        t = now;
        __builtin_amdgcn_sched_barrier(0);
    }
};
#else
struct PhaseClock {
    __device__ __forceinline__ void reset() {}
    __device__ __forceinline__ void mark(int) {}
};
#endif

// decode LDS: the CDF table, two activation buffers, head outputs, mixtures, ring
template <class Net>
struct DecLds {
    static constexpr int max_kb() {
        int m = 0;
        for (int l = 1; l < Net::kLayers; ++l) m = Net::kb(l) > m ? Net::kb(l) : m;
        return m;
    }
    static constexpr int kHS = Layout<Net>::kHeadSlots;
    static constexpr int kActBytes = max_kb() * 2 * 64 * 16;           // one layer's activations: [k-block][hi,lo][lane][16 B]
    static constexpr int kLutOff = 0;
    static constexpr int kAct0Off = (kLutEntries + 1) * 8;
    static constexpr int kAct1Off = kAct0Off + kActBytes;
    // Strides in floats, padded by one 16-byte vector: consecutive pixels (and channels) then start
    // four LDS banks apart instead of on the same bank.
    static constexpr int kHeadStride = 4 * kHS + 4;                    // head outputs of one pixel: [4 groups][kHS]
    static constexpr int kCpStride = 3 * Net::K <= 16 ? 20 : 24;       // mixture of one (pixel, channel): pi[K], mu[K], a[K]
    static constexpr int kHeadOff = kAct1Off + kActBytes;              // [16 pixels][kHeadStride] fp32, (group, register) layout
    static constexpr int kCpOff = kHeadOff + 16 * kHeadStride * 4;     // [16 pixels][3 channels][kCpStride] fp32
    // Ring of recently decoded pixels as first-layer inputs: [18 rows][2 * kRingCols columns][3] bf16.
    // Rows 0,1 are the two rows above the band.  Column c lives at slots c mod kRingCols and
    // that + kRingCols, so the values of a run of neighbour columns are always contiguous.
    // The pad keeps the 16 rows of a gather off each other's LDS banks; which pad is fastest was measured per network.
    static constexpr int kRingRowElems = 2 * Net::kRingCols * 3 + Net::kRingPad;
    static constexpr int kRingOff = kCpOff + 16 * 3 * kCpStride * 4;
    static constexpr int kMiscOff = kRingOff + 18 * kRingRowElems * 2; // ticket, abort flag
    static constexpr int kBytes = (kMiscOff + 64 + 15) / 16 * 16;
    // Two workgroups per CU have 256 registers per lane each, too few for the whole of a wave's weight slices: there
    // the biases, and the weights of the first layer and of the head where two workgroups' LDS then still fits a CU,
    // are kept in LDS behind the above and read when used.
    static constexpr int kBiasBytes = Layout<Net>::kLutOff - Layout<Net>::kWeightBytes;
    static constexpr int kFirstBytes = Net::ob(0) * Net::kb(0) * kBlockBytes;
    static constexpr int kHeadBytes = Net::ob(Net::kLayers - 1) * Net::kb(Net::kLayers - 1) * kBlockBytes;
    static constexpr bool kBiasInLds = (Net::kSharedCuLds & 1) != 0;
    static constexpr int kBiasLds = kBiasInLds ? kBiasBytes : 0;
    static constexpr bool kFirstInLds = (Net::kSharedCuLds & 2) != 0 && 2 * (kBytes + kBiasLds + kFirstBytes) <= kLdsBytes;
    static constexpr int kFirstLds = kFirstInLds ? kFirstBytes : 0;
    static constexpr bool kHeadInLds = (Net::kSharedCuLds & 4) != 0 && 2 * (kBytes + kBiasLds + kFirstLds + kHeadBytes) <= kLdsBytes;
    static constexpr int kBiasOff = kBytes;
    static constexpr int kFirstOff = kBiasOff + kBiasLds;
    static constexpr int kHeadWOff = kFirstOff + kFirstLds;
    static constexpr int kBytesShared = kHeadWOff + (kHeadInLds ? kHeadBytes : 0);
    static constexpr bool kTwoFit = 2 * kBytesShared <= kLdsBytes;      // else a CU holds one workgroup whatever the launch asks
    static_assert(kBytes % 16 == 0 && kBiasBytes % 16 == 0, "vector alignment");
    static_assert(kAct0Off % 16 == 0 && kHeadOff % 16 == 0 && kCpOff % 16 == 0, "vector alignment");
    static_assert((16 * kHS) % 16 == 0 && (kRingRowElems * 2) % 4 == 0, "vector alignment");
    // A ring row is read by the two rows below it, which trail by delay and 2 * delay columns and
    // reach two columns further back, while the column being written and the zero columns right
    // of the image are stored: all of these must be distinct slots.
    static constexpr int kMaxReach = Net::kReach1 > Net::kReach2 ? Net::kReach1 : Net::kReach2;
    // Wave w computes out-blocks w, w + 4, ... of a layer.  Where a layer's block count is not a multiple of four,
    // the last wave has a round without a block; its spare time there, in MFMAs of the other waves' chains, is
    // kIdleSlack in layer kIdleLayer (the layer where it is largest; 0: no layer has any).  The spare rounds are used to
    // fetch the pixels of the rows above the band and to write decoded pixels to the image (decode_kernel).
    static constexpr int kLastWave = kDecThreads / 64 - 1;
    static constexpr int idle_slack(int l) {
        const int nob = Net::ob(l), slots = (nob + 3) / 4;
        return kLastWave + 4 * (slots - 1) >= nob ? Net::kb(l) * (l > 0 ? 2 : 1) : 0;
    }
    static constexpr int idle_layer() {
        int best = Net::kLayers - 1;
        for (int l = 0; l < Net::kLayers; ++l) if (idle_slack(l) > idle_slack(best)) best = l;
        return best;
    }
    static constexpr int kIdleLayer = idle_layer();
    static constexpr int kIdleSlack = idle_slack(kIdleLayer);
    // Waves that idle in that round (the last ones).  With two of them the last wave, whose lanes also publish the
    // band's last two rows to the mailbox, writes the decoded pixels to the image, and the wave before it fetches:
    // the fetching wave then has loads in flight and no stores (a wave's loads and stores complete out of order with
    // each other under one counter, so a wave that has both can only wait for a load by waiting for everything).
    // With one idle wave it does both.
    static constexpr int kIdleWaves = kIdleSlack > 0 ? 4 * ((Net::ob(kIdleLayer) + 3) / 4) - Net::ob(kIdleLayer) : 0;
    static constexpr int kStoreWave = kLastWave;
    static constexpr int kFetchWave = kIdleWaves >= 2 ? kLastWave - 1 : kLastWave;
    // Does wave w have a round without an out-block in layer l?
    static constexpr bool wave_idles(int l, int w) { return w + 4 * ((Net::ob(l) + 3) / 4 - 1) >= Net::ob(l); }
    // The idle waves also have a (short) round to spare in the first layer where that is not the layer above: the
    // first, cheaper half of their jobs goes there (the fetch wave's request, the storing wave's read of the pixels).
    static constexpr bool kIdleInFirstLayer =
        kIdleSlack > 0 && kIdleLayer != 0 && wave_idles(0, kStoreWave) && wave_idles(0, kFetchWave);
    static_assert(kIdleLayer > 0 || kIdleSlack == 0, "the fetch must lie behind the barrier that follows the step's gather");
    static_assert(2 * Net::kDelay + 3 + kMaxReach <= Net::kRingCols, "ring too small for the neighbourhood");
    // what a row reads of the rows above must have been decoded in an earlier pass
    static_assert(Net::kReach1 <= Net::kDelay - 1 && Net::kReach2 <= 2 * Net::kDelay - 1, "schedule is not causal");
};

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
// stream words of two consecutive blocks of 16 sit in registers, lane j holding
// words 16 blk + j and 16 (blk + 1) + j, so a renormalisation never waits for
// memory: a pixel consumes at most three words, and the refill issued at the end
// of the step in which a block is used up is not needed for another 13 words.
struct RowReader {
    uint64_t x, y;            // the two coder states: x is the next symbol's, y the one after's (they swap per symbol)
    const uint32_t* payload;  // the row's payload: the two 8-byte states, then the words
    uint32_t last;            // index of the payload's last 32-bit word (>= 3: the states are four words)
    uint32_t nwords, pos;     // words after the state; words consumed so far
    uint32_t blk;             // block held in cur; pos >> 4 is blk or, within a step, blk + 1
    uint32_t cur, nxt;
    bool bad;
};

// Word i of the row (i counted after the state).  Indices past the end read the
// payload's last word instead: such a value is only ever consumed by a damaged
// stream, which the position check in reader_advance reports.  The load carries
// no condition, so its result can stay in flight until it is needed, and it is
// in bounds for every i as long as payload[0 .. last] is readable.
__device__ __forceinline__ uint32_t reader_word(const RowReader& rd, uint32_t i) {
    return rd.payload[min(i + 4u, rd.last)];
}

// A reader over no words at all (rows outside the image, rows whose offsets are
// damaged): `safe` is any readable pair of words; every renormalisation then counts as an over-read.
__device__ __forceinline__ void reader_init_empty(RowReader& rd, const uint32_t* safe, bool bad) {
    rd.x = kRansL; rd.y = kRansL; rd.payload = safe; rd.last = 1; rd.nwords = 0; rd.pos = 0; rd.blk = 0; rd.cur = 0; rd.nxt = 0;
    rd.bad = bad;
}

__device__ __forceinline__ void reader_init(RowReader& rd, const uint32_t* payload, uint32_t nwords_total, int j) {
    rd.x = (uint64_t)payload[0] | ((uint64_t)payload[1] << 32);
    rd.y = (uint64_t)payload[2] | ((uint64_t)payload[3] << 32);
    rd.payload = payload;
    rd.last = nwords_total - 1;
    rd.nwords = nwords_total - 4;
    rd.pos = 0;
    rd.blk = 0;
    rd.cur = reader_word(rd, (uint32_t)j);
    rd.nxt = reader_word(rd, (uint32_t)j + 16u);
    rd.bad = false;
    if (rd.x < kRansL || (rd.x >> 63)) { rd.bad = true; rd.x = kRansL; }
    if (rd.y < kRansL || (rd.y >> 63)) { rd.bad = true; rd.y = kRansL; }
}

// D(x) for the symbol found at (start, freq), and the renormalisation read.  No branches:
// the next channel's search only waits for the arithmetic, never for control flow.
// `state` is the state the symbol was coded on (rd.x for a pixel's first and third symbol, rd.y for its second).
__device__ __forceinline__ void reader_advance(RowReader& rd, uint64_t& state, uint32_t slot, uint32_t start, uint32_t freq,
                                               int j, bool active) {
    const uint32_t held = (rd.pos >> 4) != rd.blk ? rd.nxt : rd.cur;
    const uint32_t w = row_allmax((uint32_t)j == (rd.pos & 15u) ? held : 0u);   // words[pos], in every lane of the group
    const uint64_t x1 = (uint64_t)freq * (state >> 16) + slot - start;
    const bool renorm = active && x1 < kRansL;
    state = active ? (renorm ? ((x1 << 32) | w) : x1) : state;
    rd.bad = rd.bad | (renorm & (rd.pos >= rd.nwords));
    rd.pos += renorm ? 1u : 0u;
}

// After a pixel's three symbols (states x, y, x) the next symbol's state is y.
__device__ __forceinline__ void reader_next_pixel(RowReader& rd, bool active) {
    const uint64_t x = rd.x, y = rd.y;
    rd.x = active ? y : x;
    rd.y = active ? x : y;
}

// Once per step, after the pixel's three symbols: when a block has been used up, move on
// and request the block after the next.
__device__ __forceinline__ void reader_refill(RowReader& rd, int j) {
    if ((rd.pos >> 4) != rd.blk) {
        rd.blk += 1;
        rd.cur = rd.nxt;
        // scheduling only: the copy is made before the load is issued, so that the load can
        // write rd.nxt in place and stay in flight
        asm volatile("" : "+v"(rd.cur));
        rd.nxt = reader_word(rd, 16u * (rd.blk + 1u) + (uint32_t)j);
    }
}

// This wave's weight slices of one layer: out-blocks ob = wave + 4 s.  Where the
// wave has no such block (ob >= NOB) it holds a copy of the layer's last block
// and its results are discarded.
// W_LDS / B_LDS: the weights / biases stay where w / b point (a copy in LDS) and are read when used.
template <int NOB, int NKB, int SLOTS, bool W_LDS, bool B_LDS>
struct WaveLayer {
    u32x4_t a[W_LDS ? 1 : SLOTS][W_LDS ? 1 : NKB];
    f32x4_t bias[B_LDS ? 1 : SLOTS];
    const uint8_t* w_at;     // + this lane's 16 bytes
    const float* b_at;       // + this lane group's four floats
    __device__ __forceinline__ void load(const uint8_t* __restrict__ w, const float* __restrict__ b, int lane, int wave) {
        if constexpr (W_LDS) w_at = w + lane * 16;
        if constexpr (B_LDS) b_at = b + 4 * (lane >> 4);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int ob = min(wave + 4 * s, NOB - 1);
            if constexpr (!B_LDS) {
                f32x4_t t = *reinterpret_cast<const f32x4_t*>(b + 16 * ob + 4 * (lane >> 4));
                asm volatile("" : "+v"(t));      // the biases start the accumulators: in the same register file as those
                bias[s] = t;
            }
            if constexpr (!W_LDS) {
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb) {
                    u32x4_t t = *reinterpret_cast<const u32x4_t*>(w + ((ob * NKB + kb) * 64 + lane) * 16);
                    // Register allocation only: the weights, read-only MFMA operands for the whole kernel, are
                    // placed in accumulation registers, which leaves the vector registers proper to the
                    // accumulators that the vector ALU reads (no copies between the two files per block).
                    asm volatile("" : "+a"(t));
                    a[s][kb] = t;
                }
            }
        }
    }
    __device__ __forceinline__ u32x4_t A(int s, int kb, int wave) const {
        if constexpr (W_LDS) return *reinterpret_cast<const u32x4_t*>(w_at + (min(wave + 4 * s, NOB - 1) * NKB + kb) * (64 * 16));
        else return a[s][kb];
    }
    __device__ __forceinline__ f32x4_t B(int s, int wave) const {
        if constexpr (B_LDS) return *reinterpret_cast<const f32x4_t*>(b_at + 16 * min(wave + 4 * s, NOB - 1));
        else return bias[s];
    }
};

// One hidden layer on this wave's out-blocks.  Same arithmetic per output element
// as hidden_layer<> in pcc_device.h: bias, then k-blocks in order, each hi then
// lo; activation; split into hi + lo.  The out-blocks are taken one after the
// other (an accumulation chain of MFMAs issues back to back at full rate).
// In a layer's last round some waves may have no block (ob >= NOB): such a wave skips the round (a branch on
// `wave_s`, the wave's index as a scalar) and calls idle() instead, if RUN_IDLE.  Every block is finished
// (activation, split, store) inside the branch that computed it: an MFMA result is never first read behind a
// branch that the MFMA's own block does not contain.
template <int NOB, int NKB, int SLOTS, bool W_LDS, bool B_LDS, bool SPLIT_IN, bool LEAKY, bool SKIP_UNOWNED, bool RUN_IDLE,
          class Idle>
__device__ __forceinline__ void dec_hidden_layer(const WaveLayer<NOB, NKB, SLOTS, W_LDS, B_LDS>& wl, int lane, int wave,
                                                 int wave_s, const u32x4_t (&in)[NKB][2], uint8_t* __restrict__ act_out,
                                                 Idle& idle) {
    auto finish = [&](int s, const f32x4_t& acc) {
        const int ob = wave + 4 * s;
        uint32_t l0, l1;
        const uint32_t h0 = act_split_bf16<LEAKY>(acc.x, acc.y, l0);
        const uint32_t h1 = act_split_bf16<LEAKY>(acc.z, acc.w, l1);
        // out-block ob is half (ob & 1) of k-block ob/2 of the next layer's operand
        uint8_t* dst = act_out + (((ob >> 1) * 2) * 64 + lane) * 16 + 8 * (ob & 1);
        *reinterpret_cast<uint2*>(dst) = make_uint2(h0, h1);
        *reinterpret_cast<uint2*>(dst + 64 * 16) = make_uint2(l0, l1);
    };
    auto chain = [&](int s, f32x4_t& acc) {
        acc = wl.B(s, wave);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const u32x4_t a = wl.A(s, kb, wave);
            acc = mfma16(a, in[kb][0], acc);
            if (SPLIT_IN) acc = mfma16(a, in[kb][1], acc);
        }
        asm volatile("" : "+v"(acc));            // register allocation only: the result where the vector ALU reads it
    };
    constexpr bool kLastShared = 4 * (SLOTS - 1) + 3 >= NOB;      // not every wave has a block in the last round
    f32x4_t acc[SLOTS];
    if constexpr (SKIP_UNOWNED) {
        // Two workgroups per CU share the matrix cores: block after block, each finished before the next begins.
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            if (s < SLOTS - 1 || !kLastShared || wave_s + 4 * s < NOB) {
                chain(s, acc[s]);
                finish(s, acc[s]);
            } else if constexpr (RUN_IDLE) {
                idle();
            }
            __builtin_amdgcn_sched_barrier(0);      // the next block's instructions stay behind this one's
        }
    } else {
        // One workgroup per CU: the wave's blocks advance together, k-block by k-block (hi of every block, then lo of
        // every block: per output element the order stays bias, k-blocks in order, hi then lo).  A k-block's input is
        // then wanted once per SLOTS x 2 MFMAs, which is the pace at which LDS delivers the layer's input to four
        // waves reading at once; block after block, the first block's chain waited for every one of its reads.
        auto chains = [&](auto count) __attribute__((always_inline)) {
            constexpr int N = decltype(count)::value;
#pragma unroll
            for (int s = 0; s < N; ++s) acc[s] = wl.B(s, wave);
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
                for (int s = 0; s < N; ++s) acc[s] = mfma16(wl.A(s, kb, wave), in[kb][0], acc[s]);
                if (SPLIT_IN) {
#pragma unroll
                    for (int s = 0; s < N; ++s) acc[s] = mfma16(wl.A(s, kb, wave), in[kb][1], acc[s]);
                }
            }
#pragma unroll
            for (int s = 0; s < N; ++s) asm volatile("" : "+v"(acc[s]));    // register allocation only, see chain()
#pragma unroll
            for (int s = 0; s < N; ++s) finish(s, acc[s]);
        };
        if constexpr (!kLastShared) {
            chains(std::integral_constant<int, SLOTS>());
        } else if (wave_s + 4 * (SLOTS - 1) < NOB) {
            chains(std::integral_constant<int, SLOTS>());
        } else {
            chains(std::integral_constant<int, SLOTS - 1>());
            if constexpr (RUN_IDLE) idle();
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

// The whole network as seen by one wave: its weight slices of layers L .. last, and
// the per-step evaluation that hands activations from layer to layer through LDS
// (hidden layer l writes activation buffer l & 1).  Ends behind a barrier with the
// raw head outputs in `headout`.
// SHARED: the workgroup shares its CU with another (see DecLds): `lds` then holds the pieces kept there.
template <class Net, bool SHARED, int L, bool END = (L == Net::kLayers)>
struct WaveNet {
    static constexpr int NOB = Net::ob(L), NKB = Net::kb(L), SLOTS = (NOB + 3) / 4;
    static constexpr bool kHead = L == Net::kLayers - 1;
    static constexpr bool kWLds = SHARED && ((L == 0 && DecLds<Net>::kFirstInLds) || (kHead && DecLds<Net>::kHeadInLds));
    static constexpr bool kBLds = SHARED && DecLds<Net>::kBiasInLds;
    WaveLayer<NOB, NKB, SLOTS, kWLds, kBLds> wl;
    WaveNet<Net, SHARED, L + 1> rest;

    __device__ __forceinline__ void load(const uint8_t* __restrict__ model, const uint8_t* __restrict__ lds, int lane, int wave) {
        using Lay = Layout<Net>;
        using D = DecLds<Net>;
        const uint8_t* w = kWLds ? lds + (L == 0 ? D::kFirstOff : D::kHeadWOff) : model + Lay::w_off(L);
        const uint8_t* b = kBLds ? lds + D::kBiasOff + (Lay::b_off(L) - Lay::kWeightBytes) : model + Lay::b_off(L);
        wl.load(w, reinterpret_cast<const float*>(b), lane, wave);
        rest.load(model, lds, lane, wave);
    }
    // wave_s: the wave's index as a scalar (for branches); idle: what a wave without a block in the last round of
    // layer DecLds::kIdleLayer does in its place (the fetch wave is the only one that has work there).
    template <bool SKIP_UNOWNED, class Idle>
    __device__ __forceinline__ void run(const u32x4_t (&in)[NKB][2], int lane, int wave, int wave_s,
                                        uint8_t* __restrict__ act0, uint8_t* __restrict__ act1,
                                        float* __restrict__ headout, Idle& idle, PhaseClock& clk) const {
        // what waves without an out-block in this layer's last round do instead (decode_kernel says what)
        constexpr bool kRunIdle = DecLds<Net>::kIdleSlack > 0 &&
                                  (L == DecLds<Net>::kIdleLayer || (L == 0 && DecLds<Net>::kIdleInFirstLayer));
        auto idle_here = [&]() __attribute__((always_inline)) { idle(std::integral_constant<int, L>()); };
        if constexpr (kHead) {
            // registers s = 4 ob + i of group g, kept in (group, register) order; out-blocks ob = wave + 4 slot
            constexpr int HS = Layout<Net>::kHeadSlots;
#pragma unroll
            for (int slot = 0; slot < SLOTS; ++slot) {
                // a wave without a block in this round skips it; the store follows the MFMAs inside the branch
                if (4 * slot + 3 < NOB || wave_s + 4 * slot < NOB) {
                    f32x4_t acc = wl.B(slot, wave);
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb) {
                        const u32x4_t a = wl.A(slot, kb, wave);
                        acc = mfma16(a, in[kb][0], acc);
                        acc = mfma16(a, in[kb][1], acc);
                    }
                    const int ob = wave + 4 * slot;
                    *reinterpret_cast<f32x4_t*>(headout + (lane & 15) * DecLds<Net>::kHeadStride + (lane >> 4) * HS + 4 * ob) = acc;
                } else if constexpr (kRunIdle) {
                    idle_here();
                }
                if constexpr (SKIP_UNOWNED) __builtin_amdgcn_sched_barrier(0);
            }
            lds_barrier();
            clk.mark(kPhLayer0 + L);
        } else {
            uint8_t* out = (L & 1) ? act1 : act0;
            dec_hidden_layer<NOB, NKB, SLOTS, kWLds, kBLds, (L > 0), Net::kLeaky, SKIP_UNOWNED, kRunIdle>(wl, lane, wave, wave_s, in,
                                                                                                        out, idle_here);
            lds_barrier();
            clk.mark(kPhLayer0 + L);
            u32x4_t nxt[Net::kb(L + 1)][2];
            dec_load_act<Net::kb(L + 1)>(out, lane, nxt);
            // scheduling only: every read of the layer's input is issued before its first MFMA, so
            // the LDS latency is paid once per layer and not once per k-block
            __builtin_amdgcn_sched_barrier(0);
            rest.template run<SKIP_UNOWNED>(nxt, lane, wave, wave_s, act0, act1, headout, idle, clk);
        }
    }
};
template <class Net, bool SHARED, int L>
struct WaveNet<Net, SHARED, L, true> {
    __device__ __forceinline__ void load(const uint8_t* __restrict__, const uint8_t* __restrict__, int, int) {}
};

// Symbol search by the 16 lanes (j = 0..15) of one pixel: two sweeps of 16
// evaluations.  All lanes of the group return the same x, start, freq.
// prefetch(): called once the second sweep's table reads are issued; memory requests made there (the next channel's
// parameters) queue behind those reads and arrive while this channel's reductions and the coder's update run.
template <int K, class Prefetch>
__device__ __forceinline__ int group_search(const ChanParams<K>& cp, uint32_t slot, const float2* __restrict__ lut, int lane,
                                            uint32_t& start, uint32_t& freq, Prefetch& prefetch) {
    const int j = lane & 15, shift = lane & 48;
    // first sweep: Cq(16 j); lanes 0..b satisfy Cq <= slot (Cq is increasing and Cq(0) = 0).
    // Lane 0 evaluates too and discards the value: no branch.
    const uint32_t e1 = cq_eval<K>(cp, 16 * j, lut);
    const uint32_t c1 = j == 0 ? 0u : e1;
    const bool p1 = c1 <= slot;
    const int b = __popcll((__ballot(p1) >> shift) & 0xFFFFull) - 1;
    // Cq(16 b + 16), the bound of the symbol's interval if it is the block's last: it sits in lane b + 1 (65536 behind
    // the group's last lane); one lane shift brings it to lane b, which offers it to the closing minimum below.
    // (No reduction over the group is needed for it, nor for Cq(16 b): the second sweep's lane 0 evaluates that again.)
    const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(65536, (int)c1, 0x101 /* row_shl:1 */, 0xF, 0xF, false);
    const uint32_t hi_b = j == b ? up : 0xFFFFFFFFu;
    // second sweep: Cq(16 b + j)
    CqLookup<K> look;
    cq_lookup<K>(cp, 16 * b + j, lut, look);
    asm volatile("" ::: "memory");           // ordering of memory requests only: the table reads first
    prefetch();
    asm volatile("" ::: "memory");
    const uint32_t e2 = cq_finish<K>(cp, 16 * b + j, look);
    const uint32_t c2 = (b | j) == 0 ? 0u : e2;
    const bool p2 = c2 <= slot;
    const int cnt2 = __popcll((__ballot(p2) >> shift) & 0xFFFFull);
    start = row_allmax(p2 ? c2 : 0u);
    freq = row_allmin(min(p2 ? 0xFFFFFFFFu : c2, hi_b)) - start;
    return 16 * b + cnt2 - 1;
}

// N consecutive floats (N <= 16) from a 16-byte aligned LDS address, as whole vector reads.
template <int N>
__device__ __forceinline__ void lds_read_floats(const float* __restrict__ src, float (&dst)[N]) {
    constexpr int NV = (N + 3) / 4;
    f32x4_t v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = reinterpret_cast<const f32x4_t*>(src)[i];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const f32x4_t q = v[i >> 2];
        dst[i] = (i & 3) == 0 ? q.x : (i & 3) == 1 ? q.y : (i & 3) == 2 ? q.z : q.w;
    }
}

// MINBLOCKS = 1: all registers to one workgroup per CU (lowest latency per step).  MINBLOCKS = 2: two
// workgroups share a CU (some spills; a step takes about twice as long, so this only pays for jobs of
// so many bands that the work per CU, not an image's chain of steps, sets the time: launch_decode).
template <class Net, int MINBLOCKS>
__global__ void __launch_bounds__(kDecThreads, MINBLOCKS)
decode_kernel(const uint8_t* __restrict__ model, const uint8_t* __restrict__ stream, uint64_t nbytes, int n, int H,
              int W, int nbands, uint32_t dist, uint8_t* __restrict__ img_out, uint32_t* mailbox, int* status,
              uint32_t spin_limit) {
    using Lay = Layout<Net>;
    using D = DecLds<Net>;
    constexpr int K = Net::K, HS = Lay::kHeadSlots, RC = Net::kRingCols, KB0 = Net::kb(0);
    constexpr int kDelay = Net::kDelay, kMaxReach = D::kMaxReach;
    extern __shared__ __align__(16) uint8_t lds[];
    float2* lut = reinterpret_cast<float2*>(lds + D::kLutOff);
    uint8_t* act0 = lds + D::kAct0Off;
    uint8_t* act1 = lds + D::kAct1Off;
    float* headout = reinterpret_cast<float*>(lds + D::kHeadOff);
    float* cpbuf = reinterpret_cast<float*>(lds + D::kCpOff);
    uint16_t* ring = reinterpret_cast<uint16_t*>(lds + D::kRingOff);
    int* misc = reinterpret_cast<int*>(lds + D::kMiscOff);            // [0] ticket, [1] abort
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // a scalar where a branch on it pays (two workgroups per CU); measured slower as a scalar otherwise
    const int wave = MINBLOCKS > 1 ? __builtin_amdgcn_readfirstlane(tid >> 6) : tid >> 6;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);     // for branches that whole waves take
    // network role: pixel nl of the tile, k-slot group g
    const int g = lane >> 4, nl = lane & 15;
    // search role: pixel q of the band, lane j of its group
    const int q = 4 * wave + (lane >> 4), j = lane & 15;

    {
        const float2* src = reinterpret_cast<const float2*>(model + Lay::kLutOff);
        for (int i = tid; i < kLutEntries + 1; i += kDecThreads) lut[i] = src[i];
    }
    if constexpr (MINBLOCKS > 1) {
        auto stage = [&](int dst_off, int src_off, int bytes) {
            for (int i = tid * 16; i < bytes; i += kDecThreads * 16)
                *reinterpret_cast<u32x4_t*>(lds + dst_off + i) = *reinterpret_cast<const u32x4_t*>(model + src_off + i);
        };
        if constexpr (D::kBiasInLds) stage(D::kBiasOff, Lay::kWeightBytes, D::kBiasBytes);
        if constexpr (D::kFirstInLds) stage(D::kFirstOff, Lay::w_off(0), D::kFirstBytes);
        if constexpr (D::kHeadInLds) stage(D::kHeadWOff, Lay::w_off(Net::kLayers - 1), D::kHeadBytes);
    }
    // this wave's weights stay in registers (all that is not staged above), for every band the workgroup decodes
    WaveNet<Net, (MINBLOCKS > 1), 0> net;
    net.load(model, lds, lane, wave);
    const float lut_scale = *reinterpret_cast<const float*>(model + Lay::kLutScaleOff);
    const int total_bands = n * nbands;

    // network role: this lane's first-layer inputs are runs of four consecutive ring values
    // (ring row, offset within the row's window that starts at column c-2); a run the
    // network does not use reads as zero
    const uint16_t* run_ptr[KB0][2];
    bool run_used[KB0][2];
#pragma unroll
    for (int kbi = 0; kbi < KB0; ++kbi) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            int dr = 0, off = 0;
            run_used[kbi][half] = Net::run_desc(kbi, g, half, dr, off);
            run_ptr[kbi][half] = ring + (nl + 2 + dr) * D::kRingRowElems + off;
        }
    }

    // The grid has at most as many workgroups as the chip holds at once, and a workgroup decodes band after band:
    // it takes a ticket, decodes that band, takes the next.  A band only ever waits for the band above it (same
    // image), which has a smaller ticket.  Tickets come from a counter, in the order they are asked for, so every
    // ticket below a held one is held by some workgroup or finished.  With two workgroups per compute unit a
    // workgroup's first ticket is its index in the grid instead (the later ones come from the counter): the two
    // workgroups that share a unit are those of index k and k + (number of units), but they ask the counter within
    // microseconds of each other and get neighbouring tickets, so that bands which become runnable at the same time
    // share units while other units hold two workgroups that both wait (measured: 24 images of 768x512 8.2 ms; with
    // the index, the bands on a unit become runnable hundreds of steps apart, 7.3 ms).  Every ticket below a held
    // one is then still held by a workgroup that has been started, or finished: the dispatcher starts workgroups
    // in the order of their index (per die; dies run ahead of each other), and the whole grid fits the chip.
    // Should that ever not hold (a chip shared with another job's resident kernels), the bounded wait for the band
    // above ends the call with an error, not a hang.  With one workgroup per unit the counter stays: the workgroup
    // that is ready first then takes the band that can run first (a single image of 768x512: 5.52 against 5.58 ms
    // by index).  (Leaving the bands beyond the
    // resident ones to the hardware's dispatcher costs up to a third: it deals workgroups to dies and shader
    // engines in strict rotation, and waits for a place in the engine whose turn it is while others are free.)
    // Tickets are numbered band-major (band 0 of every image, then band 1 of every image, ...): the order in
    // which bands become runnable, so a workgroup holds a band that can run rather than one that waits for
    // hundreds of steps, and all images advance together.
    constexpr bool kIndexTickets = MINBLOCKS > 1;
    bool first_band = true;
    for (;;) {
    __syncthreads();                                   // the previous band's last reads of the ring and of misc
    if (tid == 0) {
        const bool stop = __hip_atomic_load(&status[kStAbort], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        misc[0] = stop ? total_bands
                       : (kIndexTickets && first_band) ? (int)blockIdx.x
                       : (kIndexTickets ? (int)gridDim.x : 0) + atomicAdd(&status[kStTicket], 1);
        misc[1] = 0;
    }
    for (int i = tid; i < 18 * D::kRingRowElems; i += kDecThreads) ring[i] = 0;
    __syncthreads();
    const int ticket = misc[0];
    first_band = false;
    if (ticket >= total_bands) break;
    const int band = ticket / n, im = ticket - band * n;

    const int r0 = band * kBandRows;
    const uint64_t rows_total = (uint64_t)n * H;
    const uint64_t table = (uint64_t)kStreamHeader + 8ull * (rows_total + 1);
    const uint64_t payload_bytes = nbytes - table;   // host guarantees nbytes >= table

    if (ticket == 0 && tid == 0) {
        const uint32_t* hdr = reinterpret_cast<const uint32_t*>(stream);
        const uint64_t last = reinterpret_cast<const uint64_t*>(stream + kStreamHeader)[rows_total];
        if (hdr[0] != kStreamMagic || hdr[1] != kStreamVersion || hdr[2] != (uint32_t)n || hdr[3] != (uint32_t)H ||
            hdr[4] != (uint32_t)W || hdr[5] != model_tag<Net>() || hdr[6] != dist || last != payload_bytes)
            set_error(status, PCC_E_STREAM);
    }

    // search role: row of this lane's pixel and its stream reader (the same in all 16 lanes of the group)
    const int qrow = r0 + q;
    const bool qrow_ok = qrow < H;
    RowReader rd;
    reader_init_empty(rd, reinterpret_cast<const uint32_t*>(stream), false);   // the stream header is always readable
    if (qrow_ok) {
        const uint64_t* offs = reinterpret_cast<const uint64_t*>(stream + kStreamHeader);
        const uint64_t rowg = (uint64_t)im * H + qrow;
        const uint64_t a = offs[rowg], b = offs[rowg + 1];
        if (a > b || b > payload_bytes || (b - a) < 16 || ((b - a) & 3) != 0 || (a & 3) != 0 ||
            (b - a) > 4ull * slab_words(W))
            rd.bad = true;
        else
            reader_init(rd, reinterpret_cast<const uint32_t*>(stream + table + a), (uint32_t)((b - a) / 4), j);
    }

    uint8_t* out_img = img_out + (size_t)im * H * W * 3;
    const uint32_t* mail_in = mailbox + ((size_t)im * nbands + (band > 0 ? band - 1 : 0)) * 2 * (size_t)W;
    uint32_t* mail_out = mailbox + ((size_t)im * nbands + band) * 2 * (size_t)W;

    const int last_row = min(r0 + kBandRows - 1, H - 1);
    const int t_begin = kDelay * r0, t_end = kDelay * last_row + W - 1;
    // The first two lanes of the fetch wave bring in the rows above the band: lane 0 row r0-2 -> ring row 0, lane 1
    // row r0-1 -> ring row 1.  That wave has a round without an out-block in one of the layers (DecLds::kIdleLayer)
    // and does the fetch there, off the path that all four waves share.
    const bool fetcher = band > 0 && tid >= D::kFetchWave * 64 && tid < D::kFetchWave * 64 + 2;
    const uint32_t* mail_row = mail_in + (size_t)(tid & 1) * W;
    // Columns right of the band's first row's column that the fetched row must be known to: row r0-2 is
    // read by the band's first row only; row r0-1 by the first row and, one delay later, by the second.
    const int ahead = (tid & 1) ? (Net::kReach1 > Net::kReach2 - kDelay ? Net::kReach1 : Net::kReach2 - kDelay)
                                : Net::kReach2;
    uint32_t pf = 0;                              // mailbox word for the next column, requested a step early

    // bf16 of the three channels of pixel word px into both copies of column cc of a ring row
    auto ring_put = [&](int rrow, int cc, uint32_t px) {
        uint16_t* d = ring + rrow * D::kRingRowElems + (cc & (RC - 1)) * 3;
        const uint16_t v0 = (uint16_t)byte_to_bf16(px & 0xFFu), v1 = (uint16_t)byte_to_bf16((px >> 8) & 0xFFu),
                       v2 = (uint16_t)byte_to_bf16((px >> 16) & 0xFFu);
        d[0] = v0; d[1] = v1; d[2] = v2;
        d[3 * RC] = v0; d[3 * RC + 1] = v1; d[3 * RC + 2] = v2;
    };
    // Bring columns 0 .. ahead of the two rows above the band into the ring, then keep
    // one column ahead: the step at t needs column (t - t_begin) + ahead.
    // wait_word: the published word of column cc (`have` if that already is one); clears ok on abort.
    auto wait_word = [&](int cc, uint32_t have, bool& ok) -> uint32_t {
        uint32_t v = have, spins = 0;
        while (!(v & kMailTag)) {
            v = __hip_atomic_load(mail_row + cc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v & kMailTag) break;
            ++spins;
            if (spins > spin_limit) { set_error(status, PCC_E_INTERNAL); ok = false; break; }
            if ((spins & 63u) == 0u &&
                __hip_atomic_load(&status[kStAbort], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                ok = false;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        return v;
    };
    auto give_up = [&]() {
        __hip_atomic_store(&status[kStAbort], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        misc[1] = 1;
    };
    if (fetcher) {
        bool ok = true;
        for (int cc = 0; cc <= ahead; ++cc) {
            if (ok && cc < W) {
                const uint32_t v = wait_word(cc, 0u, ok);
                if (ok) ring_put(tid & 1, cc, v);
            }
        }
        // Start one column further behind the band above than the data requires: the word requested a
        // step ahead has then been published when it is asked for, and is not waited for at the step's end.
        if (ok && W > ahead + 1) pf = wait_word(ahead + 1, 0u, ok);
        if (!ok) give_up();
    }
    lds_barrier();

    // Per step: the word of column (t - t_begin) + ahead + 1, requested in the step before, goes to the ring for the
    // next step's gather, and the column after it is requested; columns right of the image read as zero.  The fetch
    // wave does this where it has no out-block to compute, in two halves when it has such a round in the first layer
    // too: first the check of the word that has arrived and its conversion (fetch_check), then, behind the barrier
    // that follows this step's gather and before the one that ends the step, the ring write (fetch_put).  With those
    // two rounds the request (fetch_request) is issued at the very end of the step, after the pixel has been
    // published: the later a word is asked for, the closer the band can follow the band above (a word asked for
    // before it is published is asked for again, which holds the fetch wave up), and the load is back when the next
    // step's first layer checks it.  The request always loads (the row's last word again beyond the image): no
    // branch, the value is not used then.
    uint32_t fetched = 0;
    constexpr bool kLateRequest = D::kIdleInFirstLayer;
    auto fetch_check = [&](int t) __attribute__((always_inline)) {
        if (fetcher) {
            const int cc = t - t_begin + ahead + 1;
            uint32_t v = cc < W ? pf : 0u;
            if (cc < W && !(v & kMailTag)) {            // seldom: the band above is less than a step ahead
                bool ok = true;
                v = wait_word(cc, v, ok);
                if (!ok) give_up();
            }
            fetched = v;
        }
    };
    auto fetch_put = [&](int t) __attribute__((always_inline)) {
        if (fetcher) {
            const int cc = t - t_begin + ahead + 1;
            if (cc < W + kMaxReach) ring_put(tid & 1, cc, fetched);
            if constexpr (!kLateRequest) pf = __hip_atomic_load(mail_row + min(cc + 1, W - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    auto fetch_request = [&](int t) __attribute__((always_inline)) {
        if (fetcher) {
            const int cc = t - t_begin + ahead + 1;
            pf = __hip_atomic_load(mail_row + min(cc + 1, W - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    // The pixels decoded in step t_done go from the ring (which holds a pixel for kRingCols steps, as three bf16 of
    // its bytes) to the image: by the 16 first lanes of the storing wave, a lane per row of the band, a step later,
    // where that wave has no out-block to compute, instead of by the lanes that decoded them at the end of their
    // step, where all four waves would wait for it.  Again in two halves: the ring read, then the stores.
    uint16_t held[3] = {0, 0, 0};
    auto store_read = [&](int t_done) __attribute__((always_inline)) {
        if ((tid >> 6) == D::kStoreWave && lane < kBandRows) {
            const int cc = t_done - kDelay * (r0 + lane);
            const uint16_t* e = ring + (lane + 2) * D::kRingRowElems + (cc & (RC - 1)) * 3;
#pragma unroll
            for (int ch = 0; ch < 3; ++ch) held[ch] = e[ch];
        }
    };
    auto store_write = [&](int t_done) __attribute__((always_inline)) {
        if ((tid >> 6) == D::kStoreWave && lane < kBandRows) {
            const int row = r0 + lane, cc = t_done - kDelay * row;
            if (row < H && cc >= 0 && cc < W) {
                uint8_t* o = out_img + ((size_t)row * W + cc) * 3;
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) o[ch] = (uint8_t)(uint32_t)__uint_as_float((uint32_t)held[ch] << 16);
            }
        }
    };
    constexpr bool kStoreInIdle = D::kIdleSlack > 0;
    int t = t_begin;
    auto idle = [&](auto layer) __attribute__((always_inline)) {
        constexpr int L = decltype(layer)::value;
        if constexpr (!D::kIdleInFirstLayer) {
            fetch_check(t); fetch_put(t);
            store_read(t - 1); store_write(t - 1);
        } else if constexpr (L == 0) {
            fetch_check(t);
            store_read(t - 1);
        } else {
            fetch_put(t);
            store_write(t - 1);
        }
    };

    PhaseClock clk;
    clk.reset();
    for (; t <= t_end; ++t) {
        if ((t & 7) == 0 && misc[1] != 0) break;  // uniform: written before the last barrier; a late exit only decodes garbage
        clk.mark(kPhTop);

        // ---- gather C_ij from the ring (zeros stand for pixels outside the image); every wave builds the full tile
        u32x4_t in1[KB0][2];
        {
            const int c = t - kDelay * (r0 + nl);
            const int w0 = ((c - 2) & (RC - 1)) * 3;
            // a run is four consecutive bf16 values of a ring row (8 bytes at a 2-byte aligned address): read as two
            // dwords, which are the operand's registers as they stand
            uint32_t v[KB0][4];
#pragma unroll
            for (int kbi = 0; kbi < KB0; ++kbi) {
                uint2 lo, hi;
                __builtin_memcpy(&lo, run_ptr[kbi][0] + w0, 8);
                __builtin_memcpy(&hi, run_ptr[kbi][1] + w0, 8);
                v[kbi][0] = lo.x; v[kbi][1] = lo.y; v[kbi][2] = hi.x; v[kbi][3] = hi.y;
            }
            // one batch of LDS reads
            static_assert(KB0 == 1 || KB0 == 2, "the scheduling barrier below lists the reads explicitly");
            if constexpr (KB0 == 1)
                asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[0][2]), "+v"(v[0][3]));
            else
                asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[0][2]), "+v"(v[0][3]), "+v"(v[KB0 - 1][0]),
                                  "+v"(v[KB0 - 1][1]), "+v"(v[KB0 - 1][2]), "+v"(v[KB0 - 1][3]));
#pragma unroll
            for (int kbi = 0; kbi < KB0; ++kbi) {
                const uint32_t m0 = run_used[kbi][0] ? 0xFFFFFFFFu : 0u, m1 = run_used[kbi][1] ? 0xFFFFFFFFu : 0u;
                in1[kbi][0].x = v[kbi][0] & m0;
                in1[kbi][0].y = v[kbi][1] & m0;
                in1[kbi][0].z = v[kbi][2] & m1;
                in1[kbi][0].w = v[kbi][3] & m1;
                in1[kbi][1] = in1[kbi][0];   // unused (layer-1 inputs are exact)
            }
        }

        clk.mark(kPhGather);
        // ---- network, layers meeting in LDS
        net.template run<(MINBLOCKS > 1)>(in1, lane, wave, wave_s, act0, act1, headout, idle, clk);

        // ---- mixtures: lane j < 3K of pixel q prepares component j % K of channel j / K
        auto prepare = [&](int jj) __attribute__((always_inline)) {
            const int ch = jj / K, k = jj - K * ch;
            const float* hc = headout + q * D::kHeadStride + ch * HS;
            float pk, mk, ak;
            if constexpr (K >= 5) {
                // only this component's sigma and weight are computed (measured faster for K = 5, slower for K = 3)
                float logits[K];
                lds_read_floats<K>(hc, logits);                       // the channel's logits (for the softmax sum) ...
                const float logit_k = hc[k], mu_k = hc[K + k], ls_k = hc[2 * K + k];   // ... and this component's own three values
                channel_setup_one<K>(logits, logit_k, mu_k, ls_k, lut_scale, pk, mk, ak);
            } else {
                float raw[3 * K];
                lds_read_floats<3 * K>(hc, raw);
                ChanParams<K> all;
                channel_setup<K>(raw, lut_scale, all);
                pk = all.pi[0]; mk = all.mu[0]; ak = all.a[0];
#pragma unroll
                for (int kk = 1; kk < K; ++kk) if (k == kk) { pk = all.pi[kk]; mk = all.mu[kk]; ak = all.a[kk]; }
            }
            float* dst = cpbuf + (q * 3 + ch) * D::kCpStride + k;
            dst[0] = pk; dst[K] = mk; dst[2 * K] = ak;
        };
        if constexpr (3 * K <= 16) {
            if (j < 3 * K) prepare(j);
        } else {
            for (int jj = j; jj < 3 * K; jj += 16) prepare(jj);      // two passes for the first lanes
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");

        // What the three searches need, channel by channel: R's mixture now, G's and B's (with their coupling
        // coefficients) while the search before them waits for its last table reads.  Requested all at once, the reads
        // of the four waves keep LDS busy for hundreds of cycles in front of R's first table reads.
        ChanParams<K> cpr, cpg, cpb;
        float alpha[K], beta[K], gamma[K];
        const float* hq = headout + q * D::kHeadStride;
        // `tail` receives the last vector read, padding included: the caller keeps it in use until the values are
        // consumed (register allocation only: a padding register that is free at once is handed to the next read,
        // which then has to wait for this one)
        auto load_cp = [&](int ch, ChanParams<K>& cp, f32x4_t& tail) __attribute__((always_inline)) {
            constexpr int NV = (3 * K + 3) / 4;
            const f32x4_t* src = reinterpret_cast<const f32x4_t*>(cpbuf + (q * 3 + ch) * D::kCpStride);
            f32x4_t vv[NV];
#pragma unroll
            for (int i = 0; i < NV; ++i) vv[i] = src[i];
            tail = vv[NV - 1];
            auto at = [&](int i) { const f32x4_t w = vv[i >> 2]; return (i & 3) == 0 ? w.x : (i & 3) == 1 ? w.y : (i & 3) == 2 ? w.z : w.w; };
#pragma unroll
            for (int k = 0; k < K; ++k) { cp.pi[k] = at(k); cp.mu[k] = at(K + k); cp.a[k] = at(2 * K + k); }
        };
        f32x4_t tail_r, tail_g, tail_b;
        // coupling coefficients: canonical head outputs 9K.. (alpha), 10K.. (beta), 11K.. (gamma), wherever the head's
        // (group, register) layout put them
        auto load_g = [&]() __attribute__((always_inline)) {
            load_cp(1, cpg, tail_g);
            static_for<0, K>([&](auto kc) { alpha[decltype(kc)::value] = hq[head_slot<Net>(9 * K + decltype(kc)::value)]; });
        };
        auto load_b = [&]() __attribute__((always_inline)) {
            load_cp(2, cpb, tail_b);
            static_for<0, K>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                beta[k] = hq[head_slot<Net>(10 * K + k)];
                gamma[k] = hq[head_slot<Net>(11 * K + k)];
            });
        };
        auto load_nothing = [&]() __attribute__((always_inline)) {};
        load_cp(0, cpr, tail_r);
        asm volatile("" ::: "memory");

        clk.mark(kPhMixture);
        const int c = t - kDelay * qrow;
        const bool active = qrow_ok && c >= 0 && c < W;
        uint32_t start, freq;
        // R
        uint32_t slot = (uint32_t)rd.x & 0xFFFFu;
        const int sr = group_search<K>(cpr, slot, lut, lane, start, freq, load_g);
        reader_advance(rd, rd.x, slot, start, freq, j, active);
        float rhat = (float)sr * (1.0f / 256.0f);
        clk.mark(kPhR);
        // G given R
        asm volatile("" : "+v"(rhat) : "v"(tail_r), "v"(tail_g));    // (tied to a value known only now: stays here)
        couple_green<K>(cpg, alpha, rhat);
        slot = (uint32_t)rd.y & 0xFFFFu;
        const int sg = group_search<K>(cpg, slot, lut, lane, start, freq, load_b);
        reader_advance(rd, rd.y, slot, start, freq, j, active);
        float ghat = (float)sg * (1.0f / 256.0f);
        clk.mark(kPhG);
        // B given R, G
        asm volatile("" : "+v"(ghat) : "v"(tail_b));
        couple_blue<K>(cpb, beta, gamma, rhat, ghat);
        slot = (uint32_t)rd.x & 0xFFFFu;
        const int sb = group_search<K>(cpb, slot, lut, lane, start, freq, load_nothing);
        reader_advance(rd, rd.x, slot, start, freq, j, active);
        reader_next_pixel(rd, active);
        reader_refill(rd, j);
        clk.mark(kPhB);

        // ---- publish
        if (j == 0 && active) {
            const uint32_t px = (uint32_t)sr | ((uint32_t)sg << 8) | ((uint32_t)sb << 16);
            ring_put(q + 2, c, px);
            if (c == W - 1) {                       // the columns right of the image read as zero
#pragma unroll
                for (int z = 0; z < kMaxReach; ++z) ring_put(q + 2, W + z, 0u);
            }
            if constexpr (!kStoreInIdle) {
                uint8_t* o = out_img + ((size_t)qrow * W + c) * 3;
                o[0] = (uint8_t)sr; o[1] = (uint8_t)sg; o[2] = (uint8_t)sb;
            }
            if (q >= kBandRows - 2)
                __hip_atomic_store(mail_out + (size_t)(q - (kBandRows - 2)) * W + c, px | kMailTag, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if (c == W - 1 && (rd.bad || rd.x != kRansL || rd.y != kRansL || rd.pos != rd.nwords)) set_error(status, PCC_E_STREAM);
        }
        if constexpr (kLateRequest) fetch_request(t);
        clk.mark(kPhPublish);
        // ---- rows above the band, where no layer leaves the fetch wave spare time for it
        if constexpr (D::kIdleSlack == 0) { fetch_check(t); fetch_put(t); }
        clk.mark(kPhFetch);
        lds_barrier();
        clk.mark(kPhBarrier);
    }
#ifdef PCC_PHASE_TIMING
    if (ticket == min(kPhaseTicket, total_bands - 1) && lane == 0) {
        for (int i = 0; i < kPhCount; ++i) phase_cycles[wave][i] = clk.acc[i];
        phase_cycles[wave][kPhCount] = (unsigned long long)(t_end - t_begin + 1);
    }
#endif
    if constexpr (kStoreInIdle) { store_read(t_end); store_write(t_end); }      // the last step's pixels (the loop ended behind a barrier)
    if (misc[1] != 0) break;    // uniform: written before the last barrier.  The call has failed; no further bands.
    }
}

// ---------------------------------------------------------------------------
// test hook: full tables from given head outputs
// ---------------------------------------------------------------------------
template <class Net>
__global__ void __launch_bounds__(256)
cdf_tables_kernel(const uint8_t* __restrict__ model, const float* __restrict__ params, const uint8_t* __restrict__ rg,
                  size_t count, uint32_t* __restrict__ cq) {
    constexpr int K = Net::K, HEAD = Net::dim(Net::kLayers);
    extern __shared__ __align__(16) uint8_t lds[];
    float2* lut = reinterpret_cast<float2*>(lds);
    const float2* src = reinterpret_cast<const float2*>(model + Layout<Net>::kLutOff);
    for (int i = threadIdx.x; i < kLutEntries + 1; i += blockDim.x) lut[i] = src[i];
    __syncthreads();
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= count * 3) return;
    const size_t p = idx / 3;
    const int ch = (int)(idx - p * 3);
    const float* o = params + p * HEAD;
    float raw[3 * K];
    for (int s = 0; s < 3 * K; ++s) raw[s] = o[3 * K * ch + s];
    ChanParams<K> cp;
    channel_setup<K>(raw, *reinterpret_cast<const float*>(model + Layout<Net>::kLutScaleOff), cp);
    const float rhat = (float)rg[2 * p] * (1.0f / 256.0f), ghat = (float)rg[2 * p + 1] * (1.0f / 256.0f);
    float c1[K], c2[K];
    for (int k = 0; k < K; ++k) { c1[k] = ch == 1 ? o[9 * K + k] : o[10 * K + k]; c2[k] = o[11 * K + k]; }
    if (ch == 1) couple_green<K>(cp, c1, rhat);
    if (ch == 2) couple_blue<K>(cp, c1, c2, rhat, ghat);
    uint32_t* dst = cq + idx * 257;
    for (int e = 0; e <= 256; ++e) dst[e] = cq_full<K>(cp, e, lut);
}

// ---------------------------------------------------------------------------
// pcc_decode_static: the decoder's mailbox in an array that is part of the loaded code object, so that the call
// allocates nothing.  Each GPU the library runs on holds its own copy at its own address (resolved once per device,
// see static_scratch()); host code never uses the array's name for anything but that resolution.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = PCC_STATIC_SCRATCH_BYTES;

// Zero `count` 32-bit words (a kernel rather than a memset node: a caller may be capturing the stream).
__global__ void __launch_bounds__(256)
clear_words_kernel(uint32_t* __restrict__ dst, size_t count) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) dst[i] = 0u;
}

}  // namespace pcc

static __device__ __align__(256) uint32_t scratch[pcc::kStaticScratchBytes / 4];

// ===========================================================================
// host side
// ===========================================================================
using namespace pcc;

enum { kNetWorkload = 0, kNetPaper = 1, kNetDiagonal = 2, kNetFewerLayers = 3, kNetFewerFilters = 4, kNetMoreMixtures = 5, kNetMostMixtures = 6, kNetMoreLayers = 7, kNetMoreFilters = 8 };

struct pcc_ctx {
    int device = 0;
    int net = kNetWorkload;        // which network description the blob matched
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
    uint32_t* d_static_scratch = nullptr;   // this device's copy of the static scratch array (pcc_decode_static)
    uint32_t dist = 0;             // written to / checked against stream header word 6
    int encode_variant = 1;
    uint32_t spin_limit = 1u << 22;      // polls of a band for one pixel of the band above (seconds) before the call fails (PCC_DECODE_SPIN_LIMIT, for tests)
    int decode_variant = 0;              // 0: chosen per job; 1: one workgroup per CU; 2: two (PCC_DECODE_VARIANT, for measurements)
    // the row coder of a small job runs beside the pixel kernel, on a stream of its own
    bool overlap = true;
    uint32_t patience = kRansPatience;        // polls before a row coder beside the pixel kernel stands down
    hipStream_t side = nullptr;
    hipEvent_t ev_joined = nullptr;           // the pixel kernel's first part is done: the row coder may join
    // symbols handed from the pixel kernel to a row coder running beside it: epoch << 32 | start | (freq - 1) << 16.
    // Zero when allocated and written by nothing else, so a word carries an epoch only if that launch wrote it.
    uint64_t* d_tagged = nullptr;
    size_t tagged_count = 0;
    uint32_t epoch = 0;               // of the last launch that wrote d_tagged
    bool last_tagged = false;         // the last encode left its symbols in d_tagged, not in d_sf
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

int ensure_tagged(pcc_ctx* ctx, size_t count) {
    if (count <= ctx->tagged_count) return PCC_OK;
    if (ctx->d_tagged) { (void)hipFree(ctx->d_tagged); ctx->d_tagged = nullptr; ctx->tagged_count = 0; }
    const size_t want = count + count / 8 + 512;
    if (hipMalloc((void**)&ctx->d_tagged, want * sizeof(uint64_t)) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    if (hipMemset(ctx->d_tagged, 0, want * sizeof(uint64_t)) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    ctx->tagged_count = want;
    return PCC_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device address of this GPU's copy of `scratch`, resolved once per device with that device current (the caller
// holds a DeviceGuard).  nullptr if the runtime cannot resolve it.
constexpr int kMaxDevices = 64;
uint32_t* static_scratch(int device) {
    static std::mutex mu;
    static uint32_t* ptr[kMaxDevices] = {};
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        ptr[device] = static_cast<uint32_t*>(p);
    }
    return ptr[device];
}

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

// Calls f with a value of the network description type that `net` names.
template <class F>
auto with_net(int net, F&& f) {
    switch (net) {
        case kNetPaper: return f(NetPaper{});
        case kNetDiagonal: return f(NetDiagonal{});
        case kNetFewerLayers: return f(NetFewerLayers{});
        case kNetFewerFilters: return f(NetFewerFilters{});
        case kNetMoreMixtures: return f(NetMoreMixtures{});
        case kNetMostMixtures: return f(NetMostMixtures{});
        case kNetMoreLayers: return f(NetMoreLayers{});
        case kNetMoreFilters: return f(NetMoreFilters{});
        default: return f(NetWorkload{});
    }
}

// Does the blob header describe network Net?  (activation id 0 = ReLU, 1 = LeakyReLU 0.01)
template <class Net>
bool header_matches(const uint8_t* p) {
    if (rd32(p + 8) != (uint32_t)Net::kLayers) return false;
    for (int i = 0; i < 8; ++i)
        if (rd32(p + 12 + 4 * i) != (i <= Net::kLayers ? (uint32_t)Net::dim(i) : 0u)) return false;
    return rd32(p + 44) == (uint32_t)Net::K && rd32(p + 48) == (uint32_t)Net::kNbhd &&
           rd32(p + 52) == (uint32_t)Net::kDelay && rd32(p + 56) == (Net::kLeaky ? 1u : 0u);
}

// Weights and biases of the blob -> MFMA operand tiles in the order the kernels read them.
template <class Net>
int pack_model(const uint8_t* p, size_t blob_bytes, uint32_t dist, std::vector<uint8_t>& image) {
    using Lay = Layout<Net>;
    constexpr int NL = Net::kLayers;
    size_t need = 64;
    for (int l = 0; l < NL; ++l) need += 4 * ((size_t)Net::dim(l) * Net::dim(l + 1) + Net::dim(l + 1));
    if (blob_bytes != need) return PCC_E_BLOB;
    const uint8_t* wsrc[NL];
    const uint8_t* bsrc[NL];
    const uint8_t* q = p + 64;
    for (int l = 0; l < NL; ++l) {
        wsrc[l] = q; q += 4 * (size_t)Net::dim(l) * Net::dim(l + 1);
        bsrc[l] = q; q += 4 * (size_t)Net::dim(l + 1);
    }
    auto Wat = [&](int l, int o, int i) { return rdf(wsrc[l] + 4 * ((size_t)o * Net::dim(l) + i)); };
    auto Bat = [&](int l, int o) { return rdf(bsrc[l] + 4 * (size_t)o); };

    image.assign(Lay::kModelBytes, 0);
    uint16_t* w16 = reinterpret_cast<uint16_t*>(image.data());
    for (int l = 0; l < NL; ++l) {
        const int nob = Net::ob(l), nkb = Net::kb(l);
        const bool head = l == NL - 1;
        for (int ob = 0; ob < nob; ++ob)
            for (int kb = 0; kb < nkb; ++kb)
                for (int lane = 0; lane < 64; ++lane)
                    for (int i = 0; i < 8; ++i) {
                        const int m = lane & 15, g = lane >> 4;
                        // output feature of A row m of this out-block
                        const int o = head ? Net::head_index(m >> 2, 4 * ob + (m & 3)) : 16 * ob + m;
                        // input feature of k-slot (g, i) of this k-block
                        const int in = l == 0 ? Net::in_index(kb, g, i) : 32 * kb + kslot_feature(g, i);
                        float v = 0.0f;
                        if (o >= 0 && o < Net::dim(l + 1) && in >= 0 && in < Net::dim(l)) v = Wat(l, o, in);
                        uint16_t h;
                        if (!bf16_exact(v, &h)) return PCC_E_BLOB;
                        if (l == 0 && v != 0.0f) {
                            // fold the 1/256 input scaling into the first layer: exact unless it underflows
                            const float s = v * (1.0f / 256.0f);
                            if (!bf16_exact(s, &h) || s * 256.0f != v) return PCC_E_BLOB;
                        }
                        w16[(Lay::w_off(l) + (((ob * nkb + kb) * 64 + lane) * 16)) / 2 + i] = h;
                    }
        float* b = reinterpret_cast<float*>(image.data() + Lay::b_off(l));
        for (int s = 0; s < 16 * nob; ++s) {
            const int ob = s >> 4, m = s & 15;
            const int o = head ? Net::head_index(m >> 2, 4 * ob + (m & 3)) : s;
            b[s] = (o >= 0 && o < Net::dim(l + 1)) ? Bat(l, o) : 0.0f;
        }
    }
    // Component CDF table in units of 2^-24 so that forward differences are exact in fp32.
    float* lut = reinterpret_cast<float*>(image.data() + Lay::kLutOff);
    const double lut_scale = dist == 0 ? (double)kLutScaleGaussian : (double)kLutScaleLogistic;
    *reinterpret_cast<float*>(image.data() + Lay::kLutScaleOff) = (float)lut_scale;
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
    return PCC_OK;
}

template <class Net>
bool set_kernel_attributes() {
    constexpr int stage = std::max(params_stage_bytes<Net>(256), std::max(params_stage_bytes<Net>(512), params_stage_bytes<Net>(1024)));
    constexpr int enc = encode_model_lds_bytes<Net>() + stage, dec = DecLds<Net>::kBytes;
    static_assert(enc <= kLdsBytes && dec <= kLdsBytes && DecLds<Net>::kBytesShared <= kLdsBytes,
                  "the network does not fit a compute unit's LDS");
    bool ok = true;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<Net, 1, 512>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, enc) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<Net, 2, 512>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, enc) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<Net, 1, 1024>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, enc) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&encode_kernel<Net, 4, 256>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, enc) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<Net, 1>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, dec) == hipSuccess;
    ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<Net, 2>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, DecLds<Net>::kBytesShared) == hipSuccess;
    return ok;
}

// Workgroups of the pixel kernel.  reserve_cus: compute units left free for a kernel that runs beside it.
uint32_t encode_strips(const pcc_ctx* ctx, int W) {
    const uint32_t cols = 16u * (uint32_t)kEncodeVariants[ctx->encode_variant].tiles;
    return ((uint32_t)W + cols - 1) / cols;
}

uint32_t encode_blocks(const pcc_ctx* ctx, int n, int H, uint32_t strips, uint32_t reserve_cus) {
    const EncodeVariant ev = kEncodeVariants[ctx->encode_variant];
    const uint64_t items = (uint64_t)strips * (uint64_t)n * H;          // dims_ok: below 2^31
    const uint32_t per_block = ev.threads / 64;
    const uint64_t blocks = (items + per_block - 1) / per_block;
    const uint32_t cus = (ctx->num_cus > 0 ? (uint32_t)ctx->num_cus : 256u) - reserve_cus;
    return blocks > cus ? cus : (uint32_t)blocks;   // persistent: one workgroup per CU, looping over the items
}

// sf_tagged: see encode_kernel
template <class Net>
int launch_encode(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, uint32_t* sf, float* params, float* bits,
                  uint64_t* sf_tagged, uint32_t reserve_cus, uint32_t strip_begin, uint32_t strip_count, hipStream_t st) {
    const int kLds = encode_model_lds_bytes<Net>() + (params != nullptr ? params_stage_bytes<Net>(kEncodeVariants[ctx->encode_variant].threads) : 0);
    const uint32_t blocks = encode_blocks(ctx, n, H, strip_count, reserve_cus);
    switch (ctx->encode_variant) {
        case 0:
            hipLaunchKernelGGL((encode_kernel<Net, 1, 512>), dim3(blocks), dim3(512), kLds, st, ctx->d_model, d_img, n, H, W,
                               sf, params, bits, ctx->d_status, sf_tagged, ctx->epoch, strip_begin, strip_count);
            break;
        case 1:
            hipLaunchKernelGGL((encode_kernel<Net, 2, 512>), dim3(blocks), dim3(512), kLds, st, ctx->d_model, d_img, n, H, W,
                               sf, params, bits, ctx->d_status, sf_tagged, ctx->epoch, strip_begin, strip_count);
            break;
        case 2:
            hipLaunchKernelGGL((encode_kernel<Net, 1, 1024>), dim3(blocks), dim3(1024), kLds, st, ctx->d_model, d_img, n, H, W,
                               sf, params, bits, ctx->d_status, sf_tagged, ctx->epoch, strip_begin, strip_count);
            break;
        default:
            hipLaunchKernelGGL((encode_kernel<Net, 4, 256>), dim3(blocks), dim3(256), kLds, st, ctx->d_model, d_img, n, H, W,
                               sf, params, bits, ctx->d_status, sf_tagged, ctx->epoch, strip_begin, strip_count);
            break;
    }
    return hipGetLastError() == hipSuccess ? PCC_OK : PCC_E_HIP;
}

int launch_encode_any(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, uint32_t* sf, float* params, float* bits,
                      uint64_t* sf_tagged, uint32_t reserve_cus, uint32_t strip_begin, uint32_t strip_count, hipStream_t st) {
    return with_net(ctx->net, [&](auto net) {
        return launch_encode<decltype(net)>(ctx, d_img, n, H, W, sf, params, bits, sf_tagged, reserve_cus, strip_begin,
                                            strip_count, st);
    });
}

template <class Net>
void launch_decode(pcc_ctx* ctx, const uint8_t* d_stream, size_t nbytes, int n, int H, int W, int nbands,
                   uint8_t* d_img_out, uint32_t* d_mail, uint32_t spin_limit, hipStream_t st) {
    constexpr int kLds = DecLds<Net>::kBytes;
    const uint64_t bands = (uint64_t)n * nbands;                      // dims_ok: below 2^31
    const uint64_t cus = ctx->num_cus > 0 ? (uint64_t)ctx->num_cus : 256u;
    // One workgroup per CU decodes a step in the shortest time; two per CU take Net::kSharedStepPercent / 100 as
    // long per step when both are busy but decode twice as many bands at once.  An image is a chain of `chain`
    // steps whatever the machine does; the job is `work` band-steps.  Estimates, in percent of a step alone, fitted to
    // batches of 6 to 48 images of 768x512 in both shapes: one per CU takes the chain plus a tenth, or the work per CU
    // plus a fifth (rounds of bands that do not fill the chip); two per CU take the chain stretched by the share of
    // the time a unit's two workgroups are both busy (the work per CU over twice the chain, at most all of it), or the
    // work per place at the shared pace.  Two per CU win from about 2.2 bands per CU on (18 images of 768x512).
    const int band_rows = H < kBandRows ? H : kBandRows;
    const uint64_t chain = (uint64_t)W + (uint64_t)Net::kDelay * (H - 1);
    const uint64_t work = bands * ((uint64_t)W + (uint64_t)Net::kDelay * (band_rows - 1));
    const uint64_t per_cu = (work + cus - 1) / cus, per_half_cu = (work + 2 * cus - 1) / (2 * cus);
    const uint64_t alone = std::max(chain * 110u, per_cu * 120u);
    const uint64_t stretch = (Net::kSharedStepPercent - 113u) * std::min(per_cu, 2 * chain) / (2 * chain);
    const uint64_t shared = std::max(chain * (100u + stretch), per_half_cu * Net::kSharedStepPercent) * 103u / 100u;
    const bool two = ctx->decode_variant == 2 || (ctx->decode_variant == 0 && DecLds<Net>::kTwoFit && bands > cus && shared < alone);
    const uint32_t grid = (uint32_t)std::min(bands, two ? 2 * cus : cus);
    if (!two)
        hipLaunchKernelGGL((decode_kernel<Net, 1>), dim3(grid), dim3(kDecThreads), kLds, st, ctx->d_model, d_stream,
                           (uint64_t)nbytes, n, H, W, nbands, ctx->dist, d_img_out, d_mail, ctx->d_status, spin_limit);
    else
        hipLaunchKernelGGL((decode_kernel<Net, 2>), dim3(grid), dim3(kDecThreads), DecLds<Net>::kBytesShared, st, ctx->d_model, d_stream,
                           (uint64_t)nbytes, n, H, W, nbands, ctx->dist, d_img_out, d_mail, ctx->d_status, spin_limit);
}

inline int head_outputs(const pcc_ctx* ctx) {
    return with_net(ctx->net, [](auto net) { using Net = decltype(net); return Net::dim(Net::kLayers); });
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
        case PCC_E_SCRATCH: return "job needs more scratch memory than the library's static array holds";
        default: return "unknown error";
    }
}

size_t pcc_stream_bound(int n, int H, int W) {
    if (n < 1 || H < 1 || W < 1) return 0;
    const size_t rows = (size_t)n * H;
    return (size_t)kStreamHeader + 8 * (rows + 1) + rows * 4 * slab_words(W);
}

long pcc_wavefront_steps(int H, int W, int delay) {
    if (H < 1 || W < 1 || delay < 1) return 0;
    return (long)W + (long)delay * (H - 1);
}

int pcc_create(pcc_ctx** out, const void* h_blob, size_t blob_bytes, int hip_device) {
    if (!out || !h_blob) return PCC_E_ARG;
    *out = nullptr;
    const uint8_t* p = (const uint8_t*)h_blob;
    if (blob_bytes < 64 || rd32(p) != kBlobMagic || rd32(p + 4) != 1u) return PCC_E_BLOB;
    const uint32_t dist = rd32(p + 60);   // 0 = Gaussian mixture (Eq. (1)), 1 = logistic mixture (Eq. (8))
    if (dist > 1u) return PCC_E_BLOB;
    int net;
    if (header_matches<NetWorkload>(p)) net = kNetWorkload;
    else if (header_matches<NetPaper>(p)) net = kNetPaper;
    else if (header_matches<NetDiagonal>(p)) net = kNetDiagonal;
    else if (header_matches<NetFewerLayers>(p)) net = kNetFewerLayers;
    else if (header_matches<NetFewerFilters>(p)) net = kNetFewerFilters;
    else if (header_matches<NetMoreMixtures>(p)) net = kNetMoreMixtures;
    else if (header_matches<NetMostMixtures>(p)) net = kNetMostMixtures;
    else if (header_matches<NetMoreLayers>(p)) net = kNetMoreLayers;
    else if (header_matches<NetMoreFilters>(p)) net = kNetMoreFilters;
    else return PCC_E_BLOB;

    std::vector<uint8_t> image;
    const int prc = with_net(net, [&](auto tag) { return pack_model<decltype(tag)>(p, blob_bytes, dist, image); });
    if (prc != PCC_OK) return prc;

    DeviceGuard guard(hip_device);
    if (!guard.ok) { (void)hipGetLastError(); return PCC_E_HIP; }
    pcc_ctx* ctx = new (std::nothrow) pcc_ctx();
    if (!ctx) return PCC_E_INTERNAL;
    ctx->device = hip_device;
    ctx->net = net;
    ctx->dist = dist;
    hipDeviceProp_t prop;
    bool ok = hipGetDeviceProperties(&prop, hip_device) == hipSuccess;
    if (ok) ctx->num_cus = prop.multiProcessorCount;
    ctx->d_static_scratch = static_scratch(hip_device);
    ok = ok && ctx->d_static_scratch != nullptr;
    ok = ok && hipMalloc((void**)&ctx->d_model, image.size()) == hipSuccess;
    ok = ok && hipMalloc((void**)&ctx->d_status, kStBytes) == hipSuccess;
    ok = ok && hipMemset(ctx->d_status, 0, kStBytes) == hipSuccess;
    ok = ok && hipHostMalloc((void**)&ctx->h_status, kStBytes, hipHostMallocDefault) == hipSuccess;
    ok = ok && hipMemcpy(ctx->d_model, image.data(), image.size(), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && with_net(net, [](auto tag) { return set_kernel_attributes<decltype(tag)>(); });
    ctx->encode_variant = with_net(net, [](auto tag) { return decltype(tag)::kEncodeVariant; });
    if (const char* e = getenv("PCC_ENCODE_VARIANT")) {
        const int v = atoi(e);
        if (v >= 0 && v < 4) ctx->encode_variant = v;
    }
    // limits from the environment: negative values are taken as zero (no patience), never as huge unsigned ones
    auto env_limit = [](const char* e) { const long v = atol(e); return (uint32_t)std::min<long>(std::max<long>(v, 0), 0x7FFFFFFFl); };
    if (const char* e = getenv("PCC_DECODE_SPIN_LIMIT")) ctx->spin_limit = env_limit(e);
    if (const char* e = getenv("PCC_DECODE_VARIANT")) {
        const int v = atoi(e);
        if (v >= 0 && v <= 2) ctx->decode_variant = v;
    }
    if (const char* e = getenv("PCC_ENCODE_OVERLAP")) ctx->overlap = atoi(e) != 0;
    if (const char* e = getenv("PCC_RANS_PATIENCE")) ctx->patience = env_limit(e);
    ok = ok && hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&ctx->ev_joined, hipEventDisableTiming) == hipSuccess;
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
    if (ctx->d_tagged) (void)hipFree(ctx->d_tagged);
    if (ctx->ev_joined) (void)hipEventDestroy(ctx->ev_joined);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    delete ctx;
}

int pcc_model_info(const pcc_ctx* ctx, int* h_info) {
    if (!ctx || !h_info) return PCC_E_ARG;
    with_net(ctx->net, [&](auto tag) {
        using Net = decltype(tag);
        h_info[0] = Net::dim(Net::kLayers);
        h_info[1] = Net::K;
        h_info[2] = Net::kNbhd;
        h_info[3] = Net::kDelay;
        h_info[4] = (int)ctx->dist;
        h_info[5] = Net::kLayers;
        return 0;
    });
    return PCC_OK;
}

int pcc_encode_probs(pcc_ctx* ctx, const uint8_t* d_img, int n, int H, int W, float* d_params, float* d_bits,
                     void* hip_stream) {
    if (!ctx || !d_img || !d_params || !dims_ok(n, H, W)) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    return launch_encode_any(ctx, d_img, n, H, W, nullptr, d_params, d_bits, nullptr, 0, 0, encode_strips(ctx, W),
                             (hipStream_t)hip_stream);
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

    // A small job's row coder is a handful of workgroups, each bound by the instruction stream of its one coding wave.  It runs
    // beside the pixel kernel, on compute units the pixel kernel's grid leaves free (a pixel workgroup fills a
    // unit's LDS, so the workgroups of both kernels are resident whatever order the dispatcher takes them in),
    // and takes each symbol when it finds it written.  The row coder and what comes after it go to a stream of
    // the context's own; nothing orders that stream after the caller's, so this is only done when the caller's
    // stream is idle and the pixel kernel starts at once.  A large job's row coder needs the whole chip and
    // runs after the pixel kernel, on the caller's stream.
    const uint32_t groups = (rows + kRansRows - 1) / kRansRows;
    const uint32_t cus = ctx->num_cus > 0 ? (uint32_t)ctx->num_cus : 256u;
    bool beside = ctx->overlap && groups <= kRansBesideMaxGroups && cus >= 2 * kRansBesideMaxGroups;
    if (beside) {
        const hipError_t busy = hipStreamQuery(st);
        if (busy != hipSuccess) { (void)hipGetLastError(); beside = false; }
    }
    if (beside) {
        rc = ensure_tagged(ctx, (size_t)P * 3);
        if (rc != PCC_OK) return rc;
        if (++ctx->epoch == 0) {      // wrapped: the words of old launches would pass for new ones
            if (hipMemset(ctx->d_tagged, 0, ctx->tagged_count * sizeof(uint64_t)) != hipSuccess) return PCC_E_HIP;
            ctx->epoch = 1;
        }
    }
    ctx->last_tagged = beside;
    uint64_t* d_tagged = beside ? ctx->d_tagged : nullptr;
    // Workgroups go to the chip's eight dies in turn and stay there: a die must have room for its share of both
    // kernels, or a pixel workgroup waits for a compute unit until others of its die have ended and then works
    // through its share of the items alone.
    const uint32_t reserve = beside ? kXcds * ((groups + kXcds - 1) / kXcds) : 0u;

    if (hipMemsetAsync(ctx->d_status, 0, kStCleared, st) != hipSuccess) return PCC_E_HIP;
    prof_reset(ctx);
    const uint32_t tag = with_net(ctx->net, [](auto net) { return model_tag<decltype(net)>(); });
    auto launch_rans = [&](hipStream_t s) {
        prof_begin(ctx, PCC_T_ENCODE_RANS, s);
        if (beside)
            hipLaunchKernelGGL(rans_rows_kernel<true>, dim3(groups), dim3(kRansThreads), 0, s, d_sf, d_tagged, ctx->epoch, W,
                               rows, d_slabs, d_rw, ctx->d_status, ctx->patience);
        else
            hipLaunchKernelGGL(rans_rows_kernel<false>, dim3(groups), dim3(kRansThreads), 0, s, d_sf, d_tagged, ctx->epoch, W,
                               rows, d_slabs, d_rw, ctx->d_status, 0u);
        prof_end(ctx, PCC_T_ENCODE_RANS, s);
    };
    // what follows the row coder, and the wait for it
    auto finish = [&](hipStream_t s) -> int {
        if (rows <= kCompactScanMaxRows) {
            prof_begin(ctx, PCC_T_ENCODE_COMPACT, s);
            hipLaunchKernelGGL(compact_scan_kernel, dim3(rows), dim3(kCompactScanThreads), 0, s, d_slabs, d_rw, n, H, W, rows,
                               tag, ctx->dist, d_stream, (uint64_t)cap_bytes, ctx->d_total, ctx->d_status);
            prof_end(ctx, PCC_T_ENCODE_COMPACT, s);
        } else {
            prof_begin(ctx, PCC_T_ENCODE_SCAN, s);
            hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, d_rw, rows, n, H, W, tag, ctx->dist, d_stream, ctx->d_total);
            prof_end(ctx, PCC_T_ENCODE_SCAN, s);
            prof_begin(ctx, PCC_T_ENCODE_COMPACT, s);
            hipLaunchKernelGGL(compact_kernel, dim3(rows), dim3(64), 0, s, d_slabs, d_rw, W, rows, d_stream,
                               (uint64_t)cap_bytes, ctx->d_status);
            prof_end(ctx, PCC_T_ENCODE_COMPACT, s);
        }
        if (hipGetLastError() != hipSuccess) return PCC_E_HIP;
        if (hipMemcpyAsync(ctx->h_status, ctx->d_status, kStBytes, hipMemcpyDeviceToHost, s) != hipSuccess) return PCC_E_HIP;
        if (beside && hipMemsetAsync(ctx->d_status + kStSide, 0, 2 * sizeof(int), s) != hipSuccess) return PCC_E_HIP;
        if (hipStreamSynchronize(s) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
        return PCC_OK;
    };
    const uint32_t strips = encode_strips(ctx, W);
    if (!beside) {
        prof_begin(ctx, PCC_T_ENCODE_PIXELS, st);
        rc = launch_encode_any(ctx, d_img, n, H, W, d_sf, nullptr, nullptr, nullptr, 0, 0, strips, st);
        if (rc != PCC_OK) return rc;
        prof_end(ctx, PCC_T_ENCODE_PIXELS, st);
        launch_rans(st);
        rc = finish(st);
        if (rc != PCC_OK) return rc;
    } else {
        // An image of few rows: the row coder is the longer of the two, goes first and is in place when the pixel
        // kernel's first symbols appear.  A tall image: the pixel kernel is the longer one; it does the first
        // strips with the whole chip, and the row coder joins it (an event; the launch gap does not matter at
        // this size) for a last part sized so that both end together.  The row coder takes about as long as the
        // pixel kernel at kRansBalanceRows rows, both in proportion to the width.
        //
        // Two streams carry work from here on.  Whatever fails, the branch leaves through `drain`: both streams
        // are waited for (a row coder without its pixel kernel stands down when its patience is over), so nothing
        // still writes the caller's stream buffer or the workspace after the return, and the side status words
        // are zero again for the next call.
        auto drain = [&](int code) -> int {
            (void)hipStreamSynchronize(ctx->side);
            (void)hipStreamSynchronize(st);
            (void)hipMemsetAsync(ctx->d_status + kStSide, 0, 2 * sizeof(int), st);
            (void)hipStreamSynchronize(st);
            (void)hipGetLastError();
            return code;
        };
        const double share = 1.1 * kRansBalanceRows / rows * (double)(cus - reserve) / cus;   // of the strips, beside
        const uint32_t strips_alone = share >= 1.0 ? 0u : (uint32_t)((1.0 - share) * strips);
        if (strips_alone == 0) {
            launch_rans(ctx->side);
            prof_begin(ctx, PCC_T_ENCODE_PIXELS, st);
        } else {
            prof_begin(ctx, PCC_T_ENCODE_PIXELS, st);
            rc = launch_encode_any(ctx, d_img, n, H, W, nullptr, nullptr, nullptr, d_tagged, 0, 0, strips_alone, st);
            if (rc != PCC_OK) return drain(rc);
            if (hipEventRecord(ctx->ev_joined, st) != hipSuccess) return drain(PCC_E_HIP);
            if (hipStreamWaitEvent(ctx->side, ctx->ev_joined, 0) != hipSuccess) return drain(PCC_E_HIP);
            launch_rans(ctx->side);
        }
        rc = launch_encode_any(ctx, d_img, n, H, W, nullptr, nullptr, nullptr, d_tagged, reserve, strips_alone,
                               strips - strips_alone, st);
        if (rc != PCC_OK) return drain(rc);
        prof_end(ctx, PCC_T_ENCODE_PIXELS, st);
        rc = finish(ctx->side);
        if (rc != PCC_OK) return drain(rc);
        // the row coder ends after the pixel kernel's last store; the caller's stream is waited for as well, so
        // that the pixel kernel has retired when this returns
        if (hipStreamSynchronize(st) != hipSuccess) return drain(PCC_E_HIP);
        if (ctx->h_status[kStErr] == 0 && ctx->h_status[kStSide + kSideDefer] != 0) {
            // The row coder saw nothing of the pixel kernel for a long time and stood down: the two did not run side
            // by side.  The symbols are all there now; code them on the caller's stream.
            if (hipMemsetAsync(ctx->d_status, 0, kStCleared, st) != hipSuccess) return drain(PCC_E_HIP);
            launch_rans(st);
            rc = finish(st);
            if (rc != PCC_OK) return drain(rc);
            if (ctx->h_status[kStSide + kSideDefer] != 0) return PCC_E_INTERNAL;   // a symbol was never written
        }
    }
    prof_collect(ctx);
    if (ctx->h_status[kStErr] != 0) return ctx->h_status[kStErr];
    uint64_t total;
    memcpy(&total, ctx->h_status + kStWords, sizeof(total));
    if (total > cap_bytes) return PCC_E_CAP;
    *h_nbytes_out = (size_t)total;
    return PCC_OK;
}

// Both decoders: `d_mail` is the mailbox (zeroed here), big enough for the job.
static int decode_with_mailbox(pcc_ctx* ctx, const uint8_t* d_stream, size_t nbytes, int n, int H, int W, int nbands,
                               uint8_t* d_img_out, uint32_t* d_mail, size_t mail_bytes, bool clear_by_kernel, hipStream_t st) {
    if (clear_by_kernel) {
        const size_t words = mail_bytes / 4;
        hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<uint32_t*>(ctx->d_status),
                           kStCleared / 4);
        hipLaunchKernelGGL(clear_words_kernel, dim3((uint32_t)std::min<size_t>((words + 255) / 256, 1024)), dim3(256), 0, st,
                           d_mail, words);
        if (hipGetLastError() != hipSuccess) return PCC_E_HIP;
    } else {
        if (hipMemsetAsync(ctx->d_status, 0, kStCleared, st) != hipSuccess) return PCC_E_HIP;
        if (hipMemsetAsync(d_mail, 0, mail_bytes, st) != hipSuccess) return PCC_E_HIP;
    }
    const uint32_t spin_limit = ctx->spin_limit;
    prof_reset(ctx);
    prof_begin(ctx, PCC_T_DECODE, st);
    with_net(ctx->net, [&](auto net) {
        launch_decode<decltype(net)>(ctx, d_stream, nbytes, n, H, W, nbands, d_img_out, d_mail, spin_limit, st);
        return 0;
    });
    prof_end(ctx, PCC_T_DECODE, st);
    if (hipGetLastError() != hipSuccess) return PCC_E_HIP;
    if (hipMemcpyAsync(ctx->h_status, ctx->d_status, kStWords * sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess)
        return PCC_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) { (void)hipGetLastError(); return PCC_E_HIP; }
    prof_collect(ctx);
    return ctx->h_status[kStErr];
}

int pcc_decode(pcc_ctx* ctx, const uint8_t* d_stream, size_t nbytes, int n, int H, int W, uint8_t* d_img_out,
               void* hip_stream) {
    if (!ctx || !d_stream || !d_img_out || !dims_ok(n, H, W)) return PCC_E_ARG;
    if (((uintptr_t)d_stream & 7u) != 0) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    const uint64_t rows = (uint64_t)n * H;
    const uint64_t table = (uint64_t)kStreamHeader + 8 * (rows + 1);
    if (nbytes < table + 16 * rows) return PCC_E_STREAM;   // every row payload holds at least its two 8-byte states
    const int nbands = (H + kBandRows - 1) / kBandRows;
    const size_t mail_bytes = align_up((size_t)n * nbands * 2 * (size_t)W * 4, 256);
    int rc = ensure_workspace(ctx, mail_bytes);
    if (rc != PCC_OK) return rc;
    ctx->d_sf = nullptr; ctx->sf_count = 0;
    return decode_with_mailbox(ctx, d_stream, nbytes, n, H, W, nbands, d_img_out, reinterpret_cast<uint32_t*>(ctx->d_ws),
                               mail_bytes, false, (hipStream_t)hip_stream);
}

size_t pcc_decode_static_scratch_bytes(int n, int H, int W) {
    if (!dims_ok(n, H, W)) return 0;
    const int nbands = (H + kBandRows - 1) / kBandRows;
    return align_up((size_t)n * nbands * 2 * (size_t)W * 4, 256);
}

int pcc_decode_static(pcc_ctx* ctx, const uint8_t* d_stream, size_t nbytes, int n, int H, int W, uint8_t* d_img_out,
                      void* hip_stream) {
    if (!ctx || !d_stream || !d_img_out || !dims_ok(n, H, W)) return PCC_E_ARG;
    if (((uintptr_t)d_stream & 7u) != 0) return PCC_E_ARG;
    const size_t mail_bytes = pcc_decode_static_scratch_bytes(n, H, W);
    if (mail_bytes > kStaticScratchBytes) return PCC_E_SCRATCH;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    const uint64_t rows = (uint64_t)n * H;
    const uint64_t table = (uint64_t)kStreamHeader + 8 * (rows + 1);
    if (nbytes < table + 16 * rows) return PCC_E_STREAM;
    const int nbands = (H + kBandRows - 1) / kBandRows;
    // the array keeps the last call's words (tagged pixels of another image): the part this job uses is cleared
    return decode_with_mailbox(ctx, d_stream, nbytes, n, H, W, nbands, d_img_out, ctx->d_static_scratch, mail_bytes, true,
                               (hipStream_t)hip_stream);
}

int pcc_cdf_tables(pcc_ctx* ctx, const float* d_params, const uint8_t* d_rg, size_t count, uint32_t* d_cq,
                   void* hip_stream) {
    if (!ctx || !d_params || !d_rg || !d_cq || count == 0 || count > (1u << 26)) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    const size_t threads = count * 3;
    const dim3 grid((uint32_t)((threads + 255) / 256));
    with_net(ctx->net, [&](auto net) {
        hipLaunchKernelGGL(cdf_tables_kernel<decltype(net)>, grid, dim3(256), (kLutEntries + 1) * 8, (hipStream_t)hip_stream,
                           ctx->d_model, d_params, d_rg, count, d_cq);
        return 0;
    });
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

int pcc_copy_intervals(pcc_ctx* ctx, uint32_t* d_out, size_t count, void* hip_stream) {
    if (!ctx || !d_out) return PCC_E_ARG;
    if (!ctx->d_sf || count != ctx->sf_count) return PCC_E_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return PCC_E_HIP;
    if (ctx->last_tagged) {
        const uint32_t blocks = (uint32_t)((count + 255) / 256 < 4096 ? (count + 255) / 256 : 4096);
        hipLaunchKernelGGL(untag_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, ctx->d_tagged, count, d_out);
        return hipGetLastError() == hipSuccess ? PCC_OK : PCC_E_HIP;
    }
    if (hipMemcpyAsync(d_out, ctx->d_sf, count * sizeof(uint32_t), hipMemcpyDeviceToDevice, (hipStream_t)hip_stream) !=
        hipSuccess) return PCC_E_HIP;
    return PCC_OK;
}

#ifdef PCC_PHASE_TIMING
// measurement build only: cycles per phase and wave of the last decode's workgroup of ticket kPhaseTicket,
// h_out[4][kPhCount + 1] (the last value is the number of steps)
int pcc_debug_phase_cycles(unsigned long long* h_out) {
    return hipMemcpyFromSymbol(h_out, HIP_SYMBOL(pcc::phase_cycles), sizeof(unsigned long long) * 4 * (kPhCount + 1)) == hipSuccess
               ? PCC_OK : PCC_E_HIP;
}
#endif

}  // extern "C"
