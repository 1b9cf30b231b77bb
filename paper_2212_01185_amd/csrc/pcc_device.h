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

// ---------------------------------------------------------------------------
// Network descriptions.  Tiles are v_mfma_f32_16x16x32_bf16: out-blocks of 16
// features, k-blocks of 32 inputs; ob(l) / kb(l) are the padded block counts of
// layer l.  Two consecutive out-blocks of a hidden layer form one k-block of the
// next layer, so ob(l) = 2 kb(l+1).
// ---------------------------------------------------------------------------

// Canonical input index 3*j + ch (neighbour j in raster order, channel ch) of slot i
// (0..7) of lane group g in first-layer k-block kbi, or -1 for a padding slot, for a
// network whose byte runs carry the neighbours in place.
template <class Net>
__host__ __device__ constexpr int run_in_index(int kbi, int g, int i) {
    int dr = 0, off = 0;
    if (!Net::run_desc(kbi, g, i >> 2, dr, off)) return -1;
    const int b = off + (i & 3);
    const int len = dr == 0 ? 6 : Net::kUpBytes;
    if (b >= len) return -1;
    return (dr == -2 ? 0 : dr == -1 ? Net::kUpBytes : 2 * Net::kUpBytes) + b;
}

// The measured workloads' network: 30 -> 160 -> 160 -> 128 -> 60, ReLU, K = 5,
// neighbourhood {rows r-2, r-1 at columns c-2..c+1; row r at c-2, c-1}, wavefront delay 2.
struct NetWorkload {
    static constexpr int kLayers = 4;
    static constexpr int K = 5;
    static constexpr int kNbhd = 10, kDelay = 2;
    static constexpr int kReach1 = 1, kReach2 = 1;   // columns right of c that rows r-1 and r-2 are read at
    static constexpr int kUpBytes = 12;       // bytes of one upper row's neighbours (columns c-2..c+1)
    static constexpr int kRingCols = 8;       // decoder ring columns (power of two)
    static constexpr int kRingPad = 2;        // extra 16-bit elements per ring row
    static constexpr bool kLeaky = false;
    // Decoder with two workgroups per CU (256 registers per lane each): what of a wave's weight slices is then read
    // from a copy in LDS instead of held in registers, chosen by measurement (batches of 24 and 48 images of 768x512;
    // 24 images: none 7.21 ms, first layer 7.00, head 6.95, both 7.24, both and the biases 7.59): LDS copies cost
    // time too, so a few spilled registers can be the better deal.  1: the biases, 2: the first layer's weights,
    // 4: the head's.
    static constexpr int kEncodeVariant = 1;      // pixel kernel: two tiles per work item, 512 threads (index into the host's table)
    static constexpr int kSharedCuLds = 4;
    // Time of a decode step when both workgroups of a CU are busy, in percent of a step of a workgroup that has its
    // CU alone (measured the same way; the host chooses between the two launches with it).
    static constexpr unsigned kSharedStepPercent = 150;
    __host__ __device__ static constexpr int dim(int l) { return l == 0 ? 30 : l == 1 ? 160 : l == 2 ? 160 : l == 3 ? 128 : 60; }
    __host__ __device__ static constexpr int ob(int l) { return l == 0 ? 10 : l == 1 ? 10 : l == 2 ? 8 : 4; }
    __host__ __device__ static constexpr int kb(int l) { return l == 0 ? 1 : l == 1 ? 5 : l == 2 ? 5 : 4; }
    // Head output held by lane group g in register s = 4*out_block + i after the
    // last layer: groups 0..2 hold their channel's 15 parameters plus one coupling
    // coefficient, group 3 holds the other coupling coefficients.
    __host__ __device__ static constexpr int head_index(int g, int s) {
        return g < 3 ? (s < 15 ? 15 * g + s : (g == 1 ? 45 : (g == 2 ? 50 : -1)))
                     : (s < 4 ? 46 + s : (s < 8 ? 51 + (s - 4) : (s < 13 ? 55 + (s - 8) : -1)));
    }
    // First-layer operand: slots 0-3 (half 0) and 4-7 (half 1) of lane group g in k-block
    // kbi are four consecutive neighbour bytes of one row: row offset dr, first byte off
    // within the row's run that starts at column c-2.  Returns false for an unused half.
    __host__ __device__ static constexpr bool run_desc(int kbi, int g, int half, int& dr, int& off) {
        (void)kbi;
        if (half == 0) { dr = g < 2 ? -2 : -1; off = (g & 1) ? 8 : 0; }
        else { dr = g == 0 ? -2 : (g == 2 ? -1 : 0); off = g == 1 ? 0 : 4; }
        return true;
    }
    __host__ __device__ static constexpr int in_index(int kbi, int g, int i) { return run_in_index<NetWorkload>(kbi, g, i); }
};

// The paper's own network (Sec. III-B; hyper-parameter table of Sec. IV-E): the 12
// unmasked taps of a 5x5 first layer {rows r-2, r-1 at columns c-2..c+2; row r at c-2,
// c-1} -> 128 -> 128 -> 128 -> 128 -> 36, LeakyReLU (slope 0.01), K = 3, delay 3.
struct NetPaper {
    static constexpr int kLayers = 5;
    static constexpr int K = 3;
    static constexpr int kNbhd = 12, kDelay = 3;
    static constexpr int kReach1 = 2, kReach2 = 2;
    static constexpr int kUpBytes = 15;
    static constexpr int kRingCols = 16;
    static constexpr int kRingPad = 4;
    static constexpr bool kLeaky = true;
    static constexpr int kEncodeVariant = 1;
    static constexpr int kSharedCuLds = 4;      // 24 images of 768x512: none 8.75 ms, first layer 8.78, head 8.61, both 8.68
    static constexpr unsigned kSharedStepPercent = 145;
    __host__ __device__ static constexpr int dim(int l) { return l == 0 ? 36 : l == 5 ? 36 : 128; }
    __host__ __device__ static constexpr int ob(int l) { return l == 4 ? 3 : 8; }
    __host__ __device__ static constexpr int kb(int l) { return l == 0 ? 2 : 4; }
    // groups 0..2: the channel's 9 parameters in registers 0..8; group 1 also holds the
    // alphas and group 2 the betas in registers 9..11; group 3 holds the gammas in 0..2.
    __host__ __device__ static constexpr int head_index(int g, int s) {
        return g < 3 ? (s < 9 ? 9 * g + s : (g == 1 ? 27 + (s - 9) : (g == 2 ? 30 + (s - 9) : -1)))
                     : (s < 3 ? 33 + s : -1);
    }
    __host__ __device__ static constexpr bool run_desc(int kbi, int g, int half, int& dr, int& off) {
        if (kbi == 0) { dr = g < 2 ? -2 : -1; off = ((g & 1) ? 8 : 0) + 4 * half; return true; }
        dr = 0; off = 4 * half;
        return g == 0;
    }
    __host__ __device__ static constexpr int in_index(int kbi, int g, int i) { return run_in_index<NetPaper>(kbi, g, i); }
};

// The same network in the diagonal decoding order (Sec. III-C, Eq. (7)): a pass decodes the
// anti-diagonal r + c = t (delay 1), so the neighbours (r-2,c+2), (r-1,c+1), (r-1,c+2) are not yet
// decoded; their nine inputs carry copies of pixel (r-1,c) instead.  The copies are made by
// reading that pixel's bytes again: extra runs that start at byte 5, 6 or 8 of row r-1.
struct NetDiagonal : NetPaper {
    static constexpr int kDelay = 1;
    static constexpr int kReach1 = 0, kReach2 = 1;   // row r-1 is read up to column c, row r-2 up to c+1
    static constexpr int kRingCols = 8;
    static constexpr int kRingPad = 4;
    static constexpr unsigned kSharedStepPercent = 138;
    __host__ __device__ static constexpr bool run_desc(int kbi, int g, int half, int& dr, int& off) {
        if (kbi == 0) {
            if (g == 0) { dr = -2; off = 4 * half; }                          // row r-2, bytes 0..7
            else if (g == 1) { dr = half ? -1 : -2; off = half ? 6 : 8; }     // row r-2 bytes 8..11 | copy for (r-2,c+2)
            else if (g == 2) { dr = -1; off = 4 * half; }                     // row r-1, bytes 0..7
            else { dr = -1; off = half ? 6 : 5; }                             // copies for (r-1,c+1) | (r-1,c+2)
            return true;
        }
        if (g == 0) { dr = 0; off = 4 * half; return true; }                  // row r, bytes 0..5
        dr = -1; off = 8;                                                     // row r-1 byte 8: pixel (r-1,c), blue
        return g == 1 && half == 0;
    }
    __host__ __device__ static constexpr int in_index(int kbi, int g, int i) {
        if (kbi == 0) {
            if (g == 0) return i;
            if (g == 1) return i < 4 ? 8 + i : (i < 7 ? 12 + (i - 4) : -1);
            if (g == 2) return 15 + i;
            return i == 0 ? -1 : (i < 4 ? 24 + (i - 1) : (i < 7 ? 27 + (i - 4) : -1));
        }
        if (g == 0) return i < 6 ? 30 + i : -1;
        return (g == 1 && i == 0) ? 23 : -1;
    }
};

// The paper's network with another number of mixture components, filters or layers (the ablations of
// Sec. IV-E; wavefront order): 36 -> C -> ... -> C -> 12 K, LAYERS weight layers, LeakyReLU.  K is 3, 5
// (the head layouts above) or 7, C a multiple of 32.  The encoder keeps in LDS what fits of the packed model: six
// layers of 128 filters fit without the CDF table, of 192 filters the first two layers (the other layers' weight
// tiles and, there, the table are read from global memory).
// K = 7 (six out-blocks, 24 registers): groups 0..2 hold their channel's 21 parameters, group 3 the
// 21 coupling coefficients.
template <int MIXTURES, int C, int LAYERS>
struct NetAblation : NetPaper {
    static_assert((MIXTURES == 3 || MIXTURES == 5 || MIXTURES == 7) && C % 32 == 0 && C <= 192 && LAYERS >= 3 && LAYERS <= 7,
                  "unsupported shape");
    static constexpr int kLayers = LAYERS;
    static constexpr int K = MIXTURES;
    static constexpr int kEncodeVariant = 1;
    static constexpr int kSharedCuLds = MIXTURES >= 7 ? 7 : (MIXTURES >= 5 || LAYERS >= 6) ? 6 : NetPaper::kSharedCuLds;
    // (C = 192: a wave's weight slices alone are 264 registers; two workgroups per CU are never the better launch)
    static constexpr unsigned kSharedStepPercent = C > 128 ? 1000 : MIXTURES >= 7 ? 186 : MIXTURES >= 5 ? 153 : 147;
    __host__ __device__ static constexpr int dim(int l) { return l == 0 ? 36 : l == LAYERS ? 12 * MIXTURES : C; }
    __host__ __device__ static constexpr int ob(int l) { return (dim(l + 1) + 15) / 16; }
    __host__ __device__ static constexpr int kb(int l) { return (dim(l) + 31) / 32; }
    __host__ __device__ static constexpr int head_index(int g, int s) {
        return MIXTURES == 3 ? NetPaper::head_index(g, s)
             : MIXTURES == 5 ? NetWorkload::head_index(g, s)
                             : (s < 21 ? 21 * g + s : -1);
    }
};
using NetFewerLayers = NetAblation<3, 128, 4>;
using NetFewerFilters = NetAblation<3, 64, 5>;
using NetMoreMixtures = NetAblation<5, 128, 5>;
using NetMostMixtures = NetAblation<7, 128, 5>;
using NetMoreLayers = NetAblation<3, 128, 6>;
using NetMoreFilters = NetAblation<3, 192, 5>;

// Every canonical first-layer input sits in exactly one k-slot.
template <class Net>
constexpr bool inputs_placed_once() {
    for (int want = 0; want < Net::dim(0); ++want) {
        int n = 0;
        for (int kbi = 0; kbi < Net::kb(0); ++kbi)
            for (int g = 0; g < 4; ++g)
                for (int i = 0; i < 8; ++i) n += Net::in_index(kbi, g, i) == want ? 1 : 0;
        if (n != 1) return false;
    }
    return true;
}
static_assert(inputs_placed_once<NetWorkload>() && inputs_placed_once<NetPaper>() && inputs_placed_once<NetDiagonal>() &&
                  inputs_placed_once<NetFewerLayers>() &&
                  inputs_placed_once<NetFewerFilters>() && inputs_placed_once<NetMoreMixtures>() &&
                  inputs_placed_once<NetMostMixtures>() && inputs_placed_once<NetMoreLayers>() &&
                  inputs_placed_once<NetMoreFilters>(),
              "first-layer slot map");

constexpr int kBlockBytes = 64 * 16;  // one (out-block, k-block) A operand: 64 lanes x 8 bf16

// CDF table of the mixture's component distribution: F at z = (i - 768)/scale,
// i = 0..1536, as (value, forward difference).  scale = 128 for the Gaussian
// (|z| <= 6), 44 for the logistic of Eq. (8) (|z| <= 17.45, heavier tails).
constexpr int kLutEntries = 1537;
constexpr float kLutScaleGaussian = 128.0f;
constexpr float kLutScaleLogistic = 44.0f;
constexpr float kLutBias = 768.0f;
constexpr float kLutMax = 1536.0f;

// Packed model image: weight tiles layer by layer, fp32 biases (padded to the
// out-blocks), the CDF table, the table scale.
template <class Net>
struct Layout {
    __host__ __device__ static constexpr int w_off(int l) {
        int o = 0;
        for (int i = 0; i < l; ++i) o += Net::ob(i) * Net::kb(i) * kBlockBytes;
        return o;
    }
    static constexpr int kWeightBytes = w_off(Net::kLayers);
    __host__ __device__ static constexpr int b_off(int l) {
        int o = kWeightBytes;
        for (int i = 0; i < l; ++i) o += Net::ob(i) * 16 * 4;
        return o;
    }
    static constexpr int kLutOff = b_off(Net::kLayers);
    static constexpr int kLutScaleOff = kLutOff + (kLutEntries + 1) * 8;   // one float: table steps per unit of z
    static constexpr int kModelBytes = kLutScaleOff + 16;
    static constexpr int kHeadOB = Net::ob(Net::kLayers - 1);
    static constexpr int kHeadSlots = 4 * kHeadOB;                          // head registers per lane
    static_assert(kModelBytes % 16 == 0, "model image must be copyable in 16-byte pieces");
};
static_assert(Layout<NetWorkload>::kWeightBytes == 118784, "workload weight image size");

// Feature index (within a 32-wide k-block) held in slot i of lane group g for
// the layers after the first: the two 16-row output tiles of the previous layer,
// as MFMA left them.
__host__ __device__ constexpr int kslot_feature(int g, int i) { return 16 * (i >> 2) + 4 * g + (i & 3); }

// ---------------------------------------------------------------------------
// bf16 helpers
// ---------------------------------------------------------------------------

// Hidden activations are carried as the sum of two bf16 numbers, a ~= hi + lo with
// hi = bf16(a), lo = bf16(a - hi) (both round to nearest even): 16 significant
// bits, so that the bf16 matrix cores reproduce the fp32 network to ~1e-5
// instead of ~1e-2.  Each weight tile is multiplied with hi and then with lo.
// Applies the activation (ReLU, or LeakyReLU with slope 0.01) to two values and
// packs them: returns the hi pair, writes the lo pair.
// ReLU as a signed integer maximum of the bit pattern (negative floats are negative
// integers), LeakyReLU as the median of {a, 0.01 a, +inf}: one instruction each, where
// fmaxf() would first re-canonicalise its operand.  Inputs are finite.
template <bool LEAKY>
__device__ __forceinline__ float activation(float a) {
    if constexpr (LEAKY) return __builtin_amdgcn_fmed3f(a, 0.01f * a, __builtin_inff());
    else return __int_as_float(max(__float_as_int(a), 0));
}

template <bool LEAKY>
__device__ __forceinline__ uint32_t act_split_bf16(float a0, float a1, uint32_t& lo_pair) {
    a0 = activation<LEAKY>(a0);
    a1 = activation<LEAKY>(a1);
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

// Four bytes of a run -> four bf16 (two packed pairs): the upper halves of the fp32 conversions.
__device__ __forceinline__ void run_to_bf16(uint32_t run, uint32_t& p01, uint32_t& p23) {
    const uint32_t sel = 0x07060302u;
    p01 = __builtin_amdgcn_perm(__float_as_uint((float)((run >> 8) & 0xFFu)), __float_as_uint((float)(run & 0xFFu)), sel);
    p23 = __builtin_amdgcn_perm(__float_as_uint((float)(run >> 24)), __float_as_uint((float)((run >> 16) & 0xFFu)), sel);
}

__device__ __forceinline__ f32x4_t mfma16(u32x4_t a, u32x4_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                    __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// The network on T tiles of 16 pixels held by one wave (encoder).
//   in[t][kb][0]  layer-1 B operand of tile t (8 bf16 per lane and k-block; [1] unused)
//   out[t][ob]    raw head outputs, register s = 4*ob + i  <->  Net::head_index(lane>>4, s)
// Accumulation order per output element: bias, then k-blocks 0,1,2,..., each hi then lo.
// Activations of one layer for T tiles: [tile][k-block][0 = hi, 1 = lo].
// ---------------------------------------------------------------------------
// FAR: the weight tiles come from global memory; the reads of a k-block's tiles then stay behind the MFMAs of the
// k-block before the previous one (left to itself the compiler issues a whole layer's reads at once and spills).
template <int T, int NOB, int NKB, int OBG, bool SPLIT_IN, bool LEAKY, bool FAR = false>
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
            if constexpr (FAR) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < OBG; j += 2) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                uint32_t l0, l1, l2, l3;
                u32x4_t hi, lo;
                hi.x = act_split_bf16<LEAKY>(acc[j][t].x, acc[j][t].y, l0);
                hi.y = act_split_bf16<LEAKY>(acc[j][t].z, acc[j][t].w, l1);
                hi.z = act_split_bf16<LEAKY>(acc[j + 1][t].x, acc[j + 1][t].y, l2);
                hi.w = act_split_bf16<LEAKY>(acc[j + 1][t].z, acc[j + 1][t].w, l3);
                lo.x = l0; lo.y = l1; lo.z = l2; lo.w = l3;
                out[t][(ob0 + j) / 2][0] = hi;
                out[t][(ob0 + j) / 2][1] = lo;
            }
        }
    }
}

template <int T, int NOB, int NKB, bool FAR = false>
__device__ __forceinline__ void head_layer(const uint8_t* __restrict__ w, const float* __restrict__ bias, int lane,
                                           const u32x4_t (&in)[T][NKB][2], f32x4_t (&out)[T][NOB]) {
    const int g = lane >> 4;
    f32x4_t bv[NOB];
#pragma unroll
    for (int ob = 0; ob < NOB; ++ob) bv[ob] = *reinterpret_cast<const f32x4_t*>(bias + 16 * ob + 4 * g);
    u32x4_t a_cur[NOB], a_nxt[NOB];
#pragma unroll
    for (int ob = 0; ob < NOB; ++ob)
        a_cur[ob] = *reinterpret_cast<const u32x4_t*>(w + ((ob * NKB + 0) * 64 + lane) * 16);
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        if (kb + 1 < NKB) {
#pragma unroll
            for (int ob = 0; ob < NOB; ++ob)
                a_nxt[ob] = *reinterpret_cast<const u32x4_t*>(w + ((ob * NKB + kb + 1) * 64 + lane) * 16);
        }
#pragma unroll
        for (int ob = 0; ob < NOB; ++ob) {
#pragma unroll
            for (int t = 0; t < T; ++t) out[t][ob] = mfma16(a_cur[ob], in[t][kb][0], kb == 0 ? bv[ob] : out[t][ob]);
        }
#pragma unroll
        for (int ob = 0; ob < NOB; ++ob) {
#pragma unroll
            for (int t = 0; t < T; ++t) out[t][ob] = mfma16(a_cur[ob], in[t][kb][1], out[t][ob]);
        }
        if (kb + 1 < NKB) {
#pragma unroll
            for (int ob = 0; ob < NOB; ++ob) a_cur[ob] = a_nxt[ob];
        }
        if constexpr (FAR) __builtin_amdgcn_sched_barrier(0);
    }
}

// Layers L .. last.  WIDE selects how many out-blocks are accumulated concurrently:
// the whole layer (one tile per wave: many independent MFMA chains are needed) or two.
// `model` holds the weight tiles of the first RESIDENT layers and, straight behind them, all biases (the packed
// image itself when RESIDENT is the number of layers); the other layers' tiles are read from the image at `rest`.
template <class Net, int T, bool WIDE, int L, int RESIDENT = Net::kLayers>
__device__ __forceinline__ void mlp_from(const uint8_t* __restrict__ model, const uint8_t* __restrict__ rest, int lane,
                                         const u32x4_t (&in)[T][Net::kb(L)][2],
                                         f32x4_t (&out)[T][Layout<Net>::kHeadOB]) {
    using Lay = Layout<Net>;
    const uint8_t* w = (L < RESIDENT ? model : rest) + Lay::w_off(L);
    const float* b = reinterpret_cast<const float*>(model + Lay::w_off(RESIDENT) + (Lay::b_off(L) - Lay::kWeightBytes));
    if constexpr (L == Net::kLayers - 1) {
        head_layer<T, Net::ob(L), Net::kb(L), (L >= RESIDENT)>(w, b, lane, in, out);
    } else {
        static_assert(Net::ob(L) == 2 * Net::kb(L + 1), "two out-blocks form one k-block of the next layer");
        u32x4_t h[T][Net::kb(L + 1)][2];
        hidden_layer<T, Net::ob(L), Net::kb(L), (WIDE ? Net::ob(L) : 2), (L > 0), Net::kLeaky, (L >= RESIDENT)>(w, b, lane, in, h);
        mlp_from<Net, T, WIDE, L + 1, RESIDENT>(model, rest, lane, h, out);
    }
}

// ---------------------------------------------------------------------------
// Mixture parameters and the integer CDF (Eq. (1)-(4) of the paper).
// ---------------------------------------------------------------------------
template <int K>
struct ChanParams {
    float pi[K];   // mixture weights, softmax of the logits
    float mu[K];   // means, units of 1/256 of the grey range
    float a[K];    // table scale / sigma: table steps per unit of (edge - mu)
};

constexpr float kLog2e = 1.4426950408889634f;

// raw[0..K) logits, raw[K..2K) means, raw[2K..3K) log-sigmas of one channel.
template <int K>
__device__ __forceinline__ void channel_setup(const float (&raw)[3 * K], float lut_scale, ChanParams<K>& cp) {
    float m = raw[0];
#pragma unroll
    for (int k = 1; k < K; ++k) m = fmaxf(m, raw[k]);
    float e[K];
#pragma unroll
    for (int k = 0; k < K; ++k) e[k] = __builtin_amdgcn_exp2f((raw[k] - m) * kLog2e);
    float sum = e[0];
#pragma unroll
    for (int k = 1; k < K; ++k) sum = sum + e[k];
    const float inv = __builtin_amdgcn_rcpf(sum);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        cp.pi[k] = e[k] * inv;
        cp.mu[k] = raw[K + k];
        const float ls = fminf(fmaxf(raw[2 * K + k], -8.0f), 4.0f);   // sigma = exp(clamp(log sigma, -8, 4))
        cp.a[k] = __builtin_amdgcn_exp2f(-(ls * kLog2e)) * lut_scale;
    }
}

// One component of channel_setup: the same operations on the same inputs in the same order,
// so pi, mu, a equal cp.pi[k], cp.mu[k], cp.a[k] bit for bit.  logits[0..K) are the channel's
// logits; logit_k, mu_k, ls_k the component's own three head outputs.
template <int K>
__device__ __forceinline__ void channel_setup_one(const float (&logits)[K], float logit_k, float mu_k, float ls_k,
                                                  float lut_scale, float& pi, float& mu, float& a) {
    float m = logits[0];
#pragma unroll
    for (int k = 1; k < K; ++k) m = fmaxf(m, logits[k]);
    float e[K];
#pragma unroll
    for (int k = 0; k < K; ++k) e[k] = __builtin_amdgcn_exp2f((logits[k] - m) * kLog2e);
    float sum = e[0];
#pragma unroll
    for (int k = 1; k < K; ++k) sum = sum + e[k];
    const float inv = __builtin_amdgcn_rcpf(sum);
    pi = __builtin_amdgcn_exp2f((logit_k - m) * kLog2e) * inv;
    mu = mu_k;
    const float ls = fminf(fmaxf(ls_k, -8.0f), 4.0f);
    a = __builtin_amdgcn_exp2f(-(ls * kLog2e)) * lut_scale;
}

// Eq. (3): mu_g += alpha * r/256.   Eq. (4): mu_b += beta * r/256 + gamma * g/256.
template <int K>
__device__ __forceinline__ void couple_green(ChanParams<K>& cp, const float (&alpha)[K], float rhat) {
#pragma unroll
    for (int k = 0; k < K; ++k) cp.mu[k] = __builtin_fmaf(alpha[k], rhat, cp.mu[k]);
}
template <int K>
__device__ __forceinline__ void couple_blue(ChanParams<K>& cp, const float (&beta)[K], const float (&gamma)[K],
                                            float rhat, float ghat) {
#pragma unroll
    for (int k = 0; k < K; ++k) cp.mu[k] = __builtin_fmaf(gamma[k], ghat, __builtin_fmaf(beta[k], rhat, cp.mu[k]));
}

// Integer CDF at the lower edge of bin e (grey level e - 0.5), 1 <= e <= 255:
//   Cq(e) = e + min(floor(65280 * sum_k pi_k F(z_k)), 65280),  z_k = ((e-0.5)/256 - mu_k) / sigma_k.
// F (Phi, or the logistic CDF) is a table with linear interpolation at coordinate t = scale * z + 768,
// clamped to the table.  Entries are multiples of 2^-24 and the stored forward
// differences are exact, so one fma per lookup is non-decreasing in z; with
// pi_k >= 0 every later step (fma, floor) keeps that, hence Cq is strictly
// increasing in e and every symbol has frequency >= 1.
// In two halves, so that a caller can put other memory requests between the table reads and their use:
// cq_lookup computes the table coordinates and issues the reads, cq_finish interpolates, sums and rounds.
template <int K>
struct CqLookup {
    float t[K];
    float2 td[K];
};

template <int K>
__device__ __forceinline__ void cq_lookup(const ChanParams<K>& cp, int e, const float2* __restrict__ lut, CqLookup<K>& q) {
    const float edge = (float)(2 * e - 1) * (1.0f / 512.0f);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        q.t[k] = __builtin_amdgcn_fmed3f(__builtin_fmaf(edge - cp.mu[k], cp.a[k], kLutBias), 0.0f, kLutMax);
        q.td[k] = lut[(int)q.t[k]];                                // t >= 0: truncation is floor
    }
}

template <int K>
__device__ __forceinline__ uint32_t cq_finish(const ChanParams<K>& cp, int e, CqLookup<K>& q) {
    static_assert(K == 3 || K == 5 || K == 7, "the scheduling barrier below lists the table reads explicitly");
    float2 (&td)[K] = q.td;
    // Scheduling only: all table reads are in flight before the first is used
    // (one LDS latency per evaluation instead of K).
    if constexpr (K == 7) {
        asm volatile("" : "+v"(td[0].x), "+v"(td[0].y), "+v"(td[1].x), "+v"(td[1].y), "+v"(td[2].x), "+v"(td[2].y),
                          "+v"(td[3].x), "+v"(td[3].y), "+v"(td[4].x), "+v"(td[4].y), "+v"(td[5].x), "+v"(td[5].y),
                          "+v"(td[6].x), "+v"(td[6].y));
    } else if constexpr (K == 5) {
        asm volatile("" : "+v"(td[0].x), "+v"(td[0].y), "+v"(td[1].x), "+v"(td[1].y), "+v"(td[2].x), "+v"(td[2].y),
                          "+v"(td[3].x), "+v"(td[3].y), "+v"(td[4].x), "+v"(td[4].y));
    } else {
        asm volatile("" : "+v"(td[0].x), "+v"(td[0].y), "+v"(td[1].x), "+v"(td[1].y), "+v"(td[2].x), "+v"(td[2].y));
    }
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const float phi = __builtin_fmaf(__builtin_amdgcn_fractf(q.t[k]), td[k].y, td[k].x);
        acc = __builtin_fmaf(cp.pi[k], phi, acc);
    }
    // acc >= 0: the conversion to an unsigned integer, which drops the fraction, is the floor
    const float v = fminf(acc * 65280.0f, 65280.0f);
    return (uint32_t)e + (uint32_t)v;
}

template <int K>
__device__ __forceinline__ uint32_t cq_eval(const ChanParams<K>& cp, int e, const float2* __restrict__ lut) {
    CqLookup<K> q;
    cq_lookup<K>(cp, e, lut, q);
    return cq_finish<K>(cp, e, q);
}

template <int K>
__device__ __forceinline__ uint32_t cq_full(const ChanParams<K>& cp, int e, const float2* __restrict__ lut) {
    if (e <= 0) return 0u;
    if (e >= 256) return 65536u;
    return cq_eval<K>(cp, e, lut);
}

// ---------------------------------------------------------------------------
// rANS (one stream per image row): 64-bit state in [2^31, 2^63), 16-bit
// frequencies, 32-bit renormalisation words.
// ---------------------------------------------------------------------------
constexpr uint64_t kRansL = 1ull << 31;

}  // namespace pcc
