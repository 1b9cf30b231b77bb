// Device-side building blocks shared by the encode and decode kernels.
//
// Encoder and decoder must derive bit-identical integer CDF values for every
// pixel, otherwise decoding desynchronises.  Everything between "bytes of the
// neighbourhood" and "Cq(e)" is therefore written once, here, and compiled
// with floating-point contraction off: the same inputs go through the same
// instruction sequence in both kernels.  An MFMA output element depends only
// on its A row, its B column and the order of the k blocks, all of which are
// fixed below, so it does not matter which other pixels share a tile.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pcc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x2_t __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------
// Network shape (Sec. III-B of the paper, in the fully connected form of
// Sec. III-C): 30 -> 160 -> 160 -> 128 -> 60, padded to 32 -> ... -> 64.
// Tiles are v_mfma_f32_16x16x32_bf16: out-blocks of 16 features, k-blocks of 32.
// ---------------------------------------------------------------------------
constexpr int kL1_OB = 10, kL1_KB = 1;
constexpr int kL2_OB = 10, kL2_KB = 5;
constexpr int kL3_OB = 8, kL3_KB = 5;
constexpr int kL4_OB = 4, kL4_KB = 4;
constexpr int kBlockBytes = 64 * 16;  // one (out-block, k-block) A operand: 64 lanes x 8 bf16

// Packed model image, copied verbatim into LDS by every workgroup.
constexpr int kW1Off = 0;
constexpr int kW2Off = kW1Off + kL1_OB * kL1_KB * kBlockBytes;
constexpr int kW3Off = kW2Off + kL2_OB * kL2_KB * kBlockBytes;
constexpr int kW4Off = kW3Off + kL3_OB * kL3_KB * kBlockBytes;
constexpr int kWeightBytes = kW4Off + kL4_OB * kL4_KB * kBlockBytes;  // 118,784
constexpr int kB1Off = kWeightBytes;          // fp32 biases
constexpr int kB2Off = kB1Off + 160 * 4;
constexpr int kB3Off = kB2Off + 160 * 4;
constexpr int kB4Off = kB3Off + 128 * 4;
constexpr int kLutOff = kB4Off + 64 * 4;
// CDF table of the mixture's component distribution: F at z = (i - 768)/scale,
// i = 0..1536, as (value, forward difference).  scale = 128 for the Gaussian
// (|z| <= 6), 44 for the logistic of Eq. (8) (|z| <= 17.45, heavier tails).
constexpr int kLutEntries = 1537;
constexpr float kLutScaleGaussian = 128.0f;
constexpr float kLutScaleLogistic = 44.0f;
constexpr float kLutBias = 768.0f;
constexpr float kLutMax = 1536.0f;
constexpr int kLutScaleOff = kLutOff + (kLutEntries + 1) * 8;  // one float: table steps per unit of z
constexpr int kModelBytes = kLutScaleOff + 16;                // 133,152 (multiple of 16)
static_assert(kWeightBytes == 118784, "weight image size");
static_assert(kModelBytes % 16 == 0, "model image must be copyable in 16-byte pieces");

// Where slot i (0..7) of lane group g (0..3) of the layer-1 B operand comes
// from: row offset dr in {-2,-1,0} and byte b within that row's run of
// neighbour bytes starting at column c-2 (column c-2+b/3, channel b%3).
// Returns the canonical input index 3*j + ch, or -1 for the two padding slots.
__host__ __device__ constexpr int in1_index(int g, int i) {
    return g == 0 ? i
         : g == 1 ? (i < 4 ? 8 + i : 24 + (i - 4))
         : g == 2 ? 12 + i
                  : (i < 4 ? 20 + i : (i < 6 ? 24 + i : -1));
}
// Feature index (within a 32-wide k-block) held in slot i of lane group g for
// layers 2-4: the two 16-row output tiles of the previous layer, as MFMA left them.
__host__ __device__ constexpr int kslot_feature(int g, int i) { return 16 * (i >> 2) + 4 * g + (i & 3); }
// Head output index held by lane group g in register s = 4*out_block + i after
// the last layer: groups 0..2 hold their channel's 15 parameters plus one
// coupling coefficient, group 3 holds the other coupling coefficients.
__host__ __device__ constexpr int head_index(int g, int s) {
    return g < 3 ? (s < 15 ? 15 * g + s : (g == 1 ? 45 : (g == 2 ? 50 : -1)))
                 : (s < 4 ? 46 + s : (s < 8 ? 51 + (s - 4) : (s < 13 ? 55 + (s - 8) : -1)));
}

// ---------------------------------------------------------------------------
// bf16 helpers
// ---------------------------------------------------------------------------

// Hidden activations are carried as the sum of two bf16 numbers, a ~= hi + lo with
// hi = bf16(a), lo = bf16(a - hi) (both round to nearest even): 16 significant
// bits, so that the bf16 matrix cores reproduce the fp32 network to ~1e-5
// instead of ~1e-2.  Each weight tile is multiplied with hi and then with lo.
// Packs two ReLU'd values: returns the hi pair, writes the lo pair.
__device__ __forceinline__ uint32_t relu_split_bf16(float a0, float a1, uint32_t& lo_pair) {
    a0 = fmaxf(a0, 0.0f);
    a1 = fmaxf(a1, 0.0f);
    const f32x2_t v = {a0, a1};
    const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
    const f32x2_t r = {a0 - __uint_as_float(hi << 16), a1 - __uint_as_float(hi & 0xFFFF0000u)};
    lo_pair = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2_t));
    return hi;
}

// bf16 bit pattern of an integer 0..255 (exact).  The 1/256 input scaling is
// folded into the packed first-layer weights (a power of two, so exact).
__device__ __forceinline__ uint32_t byte_to_bf16(uint32_t x) {
    return __float_as_uint((float)x) >> 16;
}

__device__ __forceinline__ f32x4_t mfma16(u32x4_t a, u32x4_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                    __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// The network on T tiles of 16 pixels held by one wave.
//   in[t][0][0] layer-1 B operand of tile t (8 bf16 per lane)
//   out[t][ob]  raw head outputs, register s = 4*ob + i  <->  head_index(lane>>4, s)
// Accumulation order per output element: bias, then k-blocks 0,1,2,..., each hi then lo.
// ---------------------------------------------------------------------------
// Activations of one layer for T tiles: [tile][k-block][0 = hi, 1 = lo].
template <int T, int NOB, int NKB, int OBG, bool SPLIT_IN>
__device__ __forceinline__ void hidden_layer(const uint8_t* __restrict__ w, const float* __restrict__ bias,
                                             int lane, const u32x4_t (&in)[T][NKB][2],
                                             u32x4_t (&out)[T][NOB / 2][2]) {
    static_assert(NOB % OBG == 0 && OBG % 2 == 0, "out-block group must be even and divide the layer");
    const int g = lane >> 4;
#pragma unroll
    for (int ob0 = 0; ob0 < NOB; ob0 += OBG) {
        f32x4_t acc[OBG][T];
        f32x4_t bv[OBG];   // the bias is the C operand of each chain's first MFMA
#pragma unroll
        for (int j = 0; j < OBG; ++j) bv[j] = *reinterpret_cast<const f32x4_t*>(bias + 16 * (ob0 + j) + 4 * g);
        // weight tiles of the next k-block are fetched from LDS while the current ones feed the MFMAs
        u32x4_t a_cur[OBG], a_nxt[OBG];
#pragma unroll
        for (int j = 0; j < OBG; ++j)
            a_cur[j] = *reinterpret_cast<const u32x4_t*>(w + (((ob0 + j) * NKB + 0) * 64 + lane) * 16);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            if (kb + 1 < NKB) {
#pragma unroll
                for (int j = 0; j < OBG; ++j)
                    a_nxt[j] = *reinterpret_cast<const u32x4_t*>(w + (((ob0 + j) * NKB + kb + 1) * 64 + lane) * 16);
            }
#pragma unroll
            for (int j = 0; j < OBG; ++j) {
#pragma unroll
                for (int t = 0; t < T; ++t) acc[j][t] = mfma16(a_cur[j], in[t][kb][0], kb == 0 ? bv[j] : acc[j][t]);
            }
            if (SPLIT_IN) {
#pragma unroll
                for (int j = 0; j < OBG; ++j) {
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[j][t] = mfma16(a_cur[j], in[t][kb][1], acc[j][t]);
                }
            }
            if (kb + 1 < NKB) {
#pragma unroll
                for (int j = 0; j < OBG; ++j) a_cur[j] = a_nxt[j];
            }
        }
#pragma unroll
        for (int j = 0; j < OBG; j += 2) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                uint32_t l0, l1, l2, l3;
                u32x4_t hi, lo;
                hi.x = relu_split_bf16(acc[j][t].x, acc[j][t].y, l0);
                hi.y = relu_split_bf16(acc[j][t].z, acc[j][t].w, l1);
                hi.z = relu_split_bf16(acc[j + 1][t].x, acc[j + 1][t].y, l2);
                hi.w = relu_split_bf16(acc[j + 1][t].z, acc[j + 1][t].w, l3);
                lo.x = l0; lo.y = l1; lo.z = l2; lo.w = l3;
                out[t][(ob0 + j) / 2][0] = hi;
                out[t][(ob0 + j) / 2][1] = lo;
            }
        }
    }
}

template <int T>
__device__ __forceinline__ void head_layer(const uint8_t* __restrict__ w, const float* __restrict__ bias, int lane,
                                           const u32x4_t (&in)[T][kL4_KB][2], f32x4_t (&out)[T][kL4_OB]) {
    const int g = lane >> 4;
    f32x4_t bv[kL4_OB];
#pragma unroll
    for (int ob = 0; ob < kL4_OB; ++ob) bv[ob] = *reinterpret_cast<const f32x4_t*>(bias + 16 * ob + 4 * g);
    u32x4_t a_cur[kL4_OB], a_nxt[kL4_OB];
#pragma unroll
    for (int ob = 0; ob < kL4_OB; ++ob)
        a_cur[ob] = *reinterpret_cast<const u32x4_t*>(w + ((ob * kL4_KB + 0) * 64 + lane) * 16);
#pragma unroll
    for (int kb = 0; kb < kL4_KB; ++kb) {
        if (kb + 1 < kL4_KB) {
#pragma unroll
            for (int ob = 0; ob < kL4_OB; ++ob)
                a_nxt[ob] = *reinterpret_cast<const u32x4_t*>(w + ((ob * kL4_KB + kb + 1) * 64 + lane) * 16);
        }
#pragma unroll
        for (int ob = 0; ob < kL4_OB; ++ob) {
#pragma unroll
            for (int t = 0; t < T; ++t) out[t][ob] = mfma16(a_cur[ob], in[t][kb][0], kb == 0 ? bv[ob] : out[t][ob]);
        }
#pragma unroll
        for (int ob = 0; ob < kL4_OB; ++ob) {
#pragma unroll
            for (int t = 0; t < T; ++t) out[t][ob] = mfma16(a_cur[ob], in[t][kb][1], out[t][ob]);
        }
        if (kb + 1 < kL4_KB) {
#pragma unroll
            for (int ob = 0; ob < kL4_OB; ++ob) a_cur[ob] = a_nxt[ob];
        }
    }
}

// T: tiles per wave.  OBG: out-blocks accumulated concurrently (independent
// MFMA chains in flight = T * OBG).  in[t][0][0] is the layer-1 operand (exact
// bytes, no lo part).
template <int T, int OBG12, int OBG3>
__device__ __forceinline__ void mlp_forward(const uint8_t* __restrict__ model, int lane,
                                            const u32x4_t (&in)[T][1][2], f32x4_t (&out)[T][kL4_OB]) {
    u32x4_t h1[T][kL2_KB][2];
    hidden_layer<T, kL1_OB, kL1_KB, OBG12, false>(model + kW1Off, reinterpret_cast<const float*>(model + kB1Off), lane, in, h1);
    u32x4_t h2[T][kL3_KB][2];
    hidden_layer<T, kL2_OB, kL2_KB, OBG12, true>(model + kW2Off, reinterpret_cast<const float*>(model + kB2Off), lane, h1, h2);
    u32x4_t h3[T][kL4_KB][2];
    hidden_layer<T, kL3_OB, kL3_KB, OBG3, true>(model + kW3Off, reinterpret_cast<const float*>(model + kB3Off), lane, h2, h3);
    head_layer<T>(model + kW4Off, reinterpret_cast<const float*>(model + kB4Off), lane, h3, out);
}

// ---------------------------------------------------------------------------
// Mixture parameters and the integer CDF (Eq. (1)-(4) of the paper).
// ---------------------------------------------------------------------------
struct ChanParams {
    float pi[5];   // mixture weights, softmax of the logits
    float mu[5];   // means, units of 1/256 of the grey range
    float a[5];    // table scale / sigma: table steps per unit of (edge - mu)
};

constexpr float kLog2e = 1.4426950408889634f;

// raw[0..4] logits, raw[5..9] means, raw[10..14] log-sigmas of one channel.
__device__ __forceinline__ void channel_setup(const float (&raw)[15], float lut_scale, ChanParams& cp) {
    float m = raw[0];
#pragma unroll
    for (int k = 1; k < 5; ++k) m = fmaxf(m, raw[k]);
    float e[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) e[k] = __builtin_amdgcn_exp2f((raw[k] - m) * kLog2e);
    const float sum = (((e[0] + e[1]) + e[2]) + e[3]) + e[4];
    const float inv = __builtin_amdgcn_rcpf(sum);
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        cp.pi[k] = e[k] * inv;
        cp.mu[k] = raw[5 + k];
        const float ls = fminf(fmaxf(raw[10 + k], -8.0f), 4.0f);   // sigma = exp(clamp(log sigma, -8, 4))
        cp.a[k] = __builtin_amdgcn_exp2f(-(ls * kLog2e)) * lut_scale;
    }
}

// Eq. (3): mu_g += alpha * r/256.   Eq. (4): mu_b += beta * r/256 + gamma * g/256.
__device__ __forceinline__ void couple_green(ChanParams& cp, const float (&alpha)[5], float rhat) {
#pragma unroll
    for (int k = 0; k < 5; ++k) cp.mu[k] = __builtin_fmaf(alpha[k], rhat, cp.mu[k]);
}
__device__ __forceinline__ void couple_blue(ChanParams& cp, const float (&beta)[5], const float (&gamma)[5],
                                            float rhat, float ghat) {
#pragma unroll
    for (int k = 0; k < 5; ++k) cp.mu[k] = __builtin_fmaf(gamma[k], ghat, __builtin_fmaf(beta[k], rhat, cp.mu[k]));
}

// Integer CDF at the lower edge of bin e (grey level e - 0.5), 1 <= e <= 255:
//   Cq(e) = e + min(floor(65280 * sum_k pi_k Phi(z_k)), 65280),  z_k = ((e-0.5)/256 - mu_k) / sigma_k.
// F (Phi, or the logistic CDF) is a table with linear interpolation at coordinate t = scale * z + 768,
// clamped to the table.  Entries are multiples of 2^-24 and the stored forward
// differences are exact, so one fma per lookup is non-decreasing in z; with
// pi_k >= 0 every later step (fma, floor) keeps that, hence Cq is strictly
// increasing in e and every symbol has frequency >= 1.
__device__ __forceinline__ uint32_t cq_eval(const ChanParams& cp, int e, const float2* __restrict__ lut) {
    const float edge = (float)(2 * e - 1) * (1.0f / 512.0f);
    float t[5];
    float2 td[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        t[k] = __builtin_amdgcn_fmed3f(__builtin_fmaf(edge - cp.mu[k], cp.a[k], kLutBias), 0.0f, kLutMax);
        td[k] = lut[(int)t[k]];                                // t >= 0: truncation is floor
    }
    // Scheduling only: all five table reads are in flight before the first is
    // used (one LDS latency per evaluation instead of five).
    asm volatile("" : "+v"(td[0].x), "+v"(td[0].y), "+v"(td[1].x), "+v"(td[1].y), "+v"(td[2].x), "+v"(td[2].y),
                      "+v"(td[3].x), "+v"(td[3].y), "+v"(td[4].x), "+v"(td[4].y));
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        const float phi = __builtin_fmaf(__builtin_amdgcn_fractf(t[k]), td[k].y, td[k].x);
        acc = __builtin_fmaf(cp.pi[k], phi, acc);
    }
    const float v = fminf(floorf(acc * 65280.0f), 65280.0f);
    return (uint32_t)e + (uint32_t)v;
}

__device__ __forceinline__ uint32_t cq_full(const ChanParams& cp, int e, const float2* __restrict__ lut) {
    if (e <= 0) return 0u;
    if (e >= 256) return 65536u;
    return cq_eval(cp, e, lut);
}

// ---------------------------------------------------------------------------
// rANS (one stream per image row): 64-bit state in [2^31, 2^63), 16-bit
// frequencies, 32-bit renormalisation words.
// ---------------------------------------------------------------------------
constexpr uint64_t kRansL = 1ull << 31;

}  // namespace pcc
