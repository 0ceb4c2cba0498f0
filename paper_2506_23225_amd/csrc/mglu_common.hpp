// Shared definitions of the MGLU kernels for gfx950: packed-format constants,
// MFMA fragment traits and the fused epilogue (Eq. 3 of the paper).
//
// Packed formats (both produced by mglu_pack.hip, consumed by the kernels)
// -----------------------------------------------------------------------
// The logical weight matrix W[k][j] (k < d_model, j < d_ff) is cut into column
// blocks of 16 (index jb) and reduction chunks of 128 (index kc), zero-padded to
// those multiples.  One (jb, kc) pair is a "chunk": 16 x 128 elements.
//
//   bf16 weights  [jb][kc][tile t<4][lane<64][e<8]  : W[128kc + 32t + 8(lane/16) + e][16jb + lane%16]
//   fp32 weights  [jb][kc][tile t<8][lane<64][e<4]  : W[128kc + 16t + 4(lane/16) + e][16jb + lane%16]
//
// so that one wavefront load of 16 bytes per lane is a contiguous 1 KiB run and
// lands directly in the A-operand layout of v_mfma_f32_16x16x32_bf16 (row =
// lane%16, eight consecutive k per lane) or, for fp32, of four
// v_mfma_f32_16x16x4_f32 (row = lane%16, k = lane/16, one per e).
//
//   masks  [jb][kc][lane<64][word<NMP]  uint32,  NMP = n_masks rounded up to 1,2,4,8,16
//          (NMP >= 8: [jb][kc][piece<NMP/4][lane<64][word<4], word w of a lane = piece w/4, word w%4,
//           so that every 16-byte-per-lane load of a wavefront is one contiguous 1 KiB run)
//
// A lane's NMP words hold the NMP x 32 mask bits of the 32 weight elements that
// lane holds in the chunk.  16-bit elements: they form 16 register pairs (tile t, pair p = e/2; low
// half e even, high half e odd); the bit for (t, p, mask i, half hf) is in word
// Half16Common::mask_word(t, p, i) at position mask_bit(t, p, i) + 16*hf, so one shift brings both
// bits of a pair to the two sign positions 15 and 31.  For 2 to 16 masks the words are
// assigned so that registers p and p + 2 of a fragment find their bits in two neighbouring words at
// the same position: one 64-bit shift then serves both.  16 masks (16-bit elements) are two 8-mask
// halves side by side: words 0-7 of a lane (pieces 0, 1) are masks 0-7 in the 8-mask order, words
// 8-15 (pieces 2, 3) masks 8-15 -- a kernel built for 8 masks can read either half on its own
// (chunk stride 4 KiB, half h at byte 2048 h), which is how the MFMA-tiled kernel runs 16 masks.
// fp32: element E = 4t + e, linear = E*NMP + i -> word linear/32, bit linear%32.
//
//   planar masks  [jb][mask i < n_masks][kc][lane<64]  uint32
//
// the second mask format, for the routed kernel that reads only the selected masks: a word holds the
// 32 bits of one mask for the 32 elements of its lane (bit = Traits::planar_bit(t, e)), and the words
// of one mask of one column block are one contiguous run over the chunks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mglu {

constexpr int kColBlock = 16;   // output columns per MFMA tile
constexpr int kChunkK = 128;    // reduction elements per chunk
constexpr int kWave = 64;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// element types of x, W and out
enum Elem { kElemF32 = 0, kElemBf16 = 1, kElemF16 = 2 };

constexpr int kMaxMasks = 16;
__host__ __device__ constexpr int round_up_masks(int n) { return n <= 1 ? 1 : n <= 2 ? 2 : n <= 4 ? 4 : n <= 8 ? 8 : 16; }
__host__ __device__ constexpr long ceil_div(long a, long b) { return (a + b - 1) / b; }

// Byte offset of a lane's mask words inside a chunk's mask block, and the stride between its
// 16-byte pieces when there are 8 or 16 masks.
template <int NMP>
__host__ __device__ constexpr uint32_t mask_lane_bytes(int lane) { return NMP >= 8 ? lane * 16 : lane * NMP * 4; }
constexpr uint32_t kMaskPieceBytes = kWave * 16;

// ---- fp32 <-> bf16 ---------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round to nearest, ties to even; NaN stays NaN (the hardware's packed conversion, one instruction
// for two values where the compiler can pair them)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

// fp16 (IEEE binary16), the paper's own precision: hardware conversions, round to nearest even
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b) { return (float)__builtin_bit_cast(_Float16, (uint16_t)b); }
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// ---- Swish, beta = 1:  z * sigmoid(z) = z / (1 + exp(-z)) --------------------------------
__device__ __forceinline__ float swish(float z)
{
    // exp(-z) overflows to +inf for z < -88 and the product is then -0, the right limit.  The
    // reciprocal is the hardware's (1 ulp): a correctly rounded quotient costs ten more instructions
    // per element and buys nothing at the layer's tolerances.
    return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z));
}

// ---- element traits ------------------------------------------------------------------------
// A chunk is TILES fragments per lane; a fragment is 16 bytes of W (A operand) or x (B operand).
// 64-bit left shift as one instruction.  Written as assembly because the compiler, seeing that only
// two bits of each half are used afterwards, narrows the C expression back to two 32-bit shifts.
__device__ __forceinline__ uint64_t shl64(uint64_t v, int s)
{
    uint64_t r;
    asm("v_lshlrev_b64 %0, %1, %2" : "=v"(r) : "s"(s), "v"(v));
    return r;
}

// 16-bit elements, two to a register.  bf16 and fp16 share the fragment shapes and -- the sign bit
// being bit 15 of either format -- the mask application; they differ in the MFMA and the rounding.
struct Half16Common {
    typedef u32x4 frag;                       // 4 registers, each a (k, k+1) pair of elements
    static constexpr int TILES = 4;           // 32 k per tile
    static constexpr int TILE_K = 32;
    static constexpr int LANE_K = 8;          // consecutive k one lane holds per tile
    static constexpr int ELEM_BYTES = 2;

    // W fragment of tile t with the sign of every element whose bit in mask i is set flipped.
    // `i` may be a compile-time constant or a run-time value that is uniform over the wavefront
    // (the word that holds a bit does not depend on i, only the shift does).
    // With 8 or 16 masks two registers of the fragment take their bits from two neighbouring words
    // at the same shift, so one 64-bit shift (full rate on gfx950) serves both: 6 vector-ALU
    // instructions per fragment and mask instead of 8.
    template <int NMP>
    __device__ static __forceinline__ frag flip(frag w, const uint32_t (&m)[NMP], int t, int i)
    {
        frag r;
        if constexpr (NMP == 8) {
            // pair p: word 2t + p/2, bit (p%2)*8 + i
            const uint64_t mm = ((uint64_t)m[2 * t + 1] << 32) | m[2 * t];
            const uint64_t a = shl64(mm, 15 - i), b = shl64(mm, 7 - i);
            r[0] = w[0] ^ ((uint32_t)a & 0x80008000u);
            r[1] = w[1] ^ ((uint32_t)b & 0x80008000u);
            r[2] = w[2] ^ ((uint32_t)(a >> 32) & 0x80008000u);
            r[3] = w[3] ^ ((uint32_t)(b >> 32) & 0x80008000u);
        } else if constexpr (NMP == 16) {
            // two 8-mask halves side by side: mask i lives in words [8 (i/8), 8 (i/8) + 8) in the 8-mask order
            const int o = 8 * (i >> 3) + 2 * t, s = i & 7;
            const uint64_t mm = ((uint64_t)m[o + 1] << 32) | m[o];
            const uint64_t a = shl64(mm, 15 - s), b = shl64(mm, 7 - s);
            r[0] = w[0] ^ ((uint32_t)a & 0x80008000u);
            r[1] = w[1] ^ ((uint32_t)b & 0x80008000u);
            r[2] = w[2] ^ ((uint32_t)(a >> 32) & 0x80008000u);
            r[3] = w[3] ^ ((uint32_t)(b >> 32) & 0x80008000u);
        } else if constexpr (NMP == 4) {
            // pair p: word 2(t/2) + p/2, bit ((t%2)*2 + p%2)*4 + i
            const uint64_t mm = ((uint64_t)m[2 * (t / 2) + 1] << 32) | m[2 * (t / 2)];
            const uint64_t a = shl64(mm, 15 - ((t % 2) * 8 + i)), b = shl64(mm, 15 - ((t % 2) * 8 + 4 + i));
            r[0] = w[0] ^ ((uint32_t)a & 0x80008000u);
            r[1] = w[1] ^ ((uint32_t)b & 0x80008000u);
            r[2] = w[2] ^ ((uint32_t)(a >> 32) & 0x80008000u);
            r[3] = w[3] ^ ((uint32_t)(b >> 32) & 0x80008000u);
        } else if constexpr (NMP == 2) {
            // pair p: word p/2, bit (t*2 + p%2)*2 + i
            const uint64_t mm = ((uint64_t)m[1] << 32) | m[0];
            const uint64_t a = shl64(mm, 15 - (t * 4 + i)), b = shl64(mm, 15 - (t * 4 + 2 + i));
            r[0] = w[0] ^ ((uint32_t)a & 0x80008000u);
            r[1] = w[1] ^ ((uint32_t)b & 0x80008000u);
            r[2] = w[2] ^ ((uint32_t)(a >> 32) & 0x80008000u);
            r[3] = w[3] ^ ((uint32_t)(b >> 32) & 0x80008000u);
        } else {
            // one mask: pair p of tile t at bit 4t + p of the only word
#pragma unroll
            for (int p = 0; p < 4; ++p) r[p] = w[p] ^ ((m[0] << (15 - (4 * t + p) - i)) & 0x80008000u);
        }
        return r;
    }
    // Where the pack kernel puts the bit of (tile t, pair p, mask i) of a lane: word index and bit
    // position inside the low half of that word (the high half holds the pair's second element).
    template <int NMP>
    __host__ __device__ static constexpr int mask_word(int t, int p, int i)
    {
        return NMP == 16 ? 8 * (i / 8) + 2 * t + p / 2
             : NMP == 8  ? 2 * t + p / 2
             : NMP == 4  ? 2 * (t / 2) + p / 2
             : NMP == 2  ? p / 2
                         : 0;
    }
    template <int NMP>
    __host__ __device__ static constexpr int mask_bit(int t, int p, int i)
    {
        return NMP == 16 ? (p % 2) * 8 + i % 8
             : NMP == 8  ? (p % 2) * 8 + i
             : NMP == 4  ? ((t % 2) * 2 + p % 2) * 4 + i
             : NMP == 2  ? (t * 2 + p % 2) * 2 + i
                         : 4 * t + p;
    }
    // The same with a mask index that is only known at run time (uniform over the wavefront).  Below 16
    // masks the word that holds a bit does not depend on i, only the shift does; with 16 the half is
    // selected first.
    template <int NMP>
    __device__ static __forceinline__ frag flip_at(frag w, const uint32_t (&m)[NMP], int t, int i)
    {
        if constexpr (NMP == 16) {
            const bool hi = i >= 8;
            const uint32_t half[8] = {hi ? m[8] : m[0],  hi ? m[9] : m[1],  hi ? m[10] : m[2], hi ? m[11] : m[3],
                                      hi ? m[12] : m[4], hi ? m[13] : m[5], hi ? m[14] : m[6], hi ? m[15] : m[7]};
            return flip<8>(w, half, t, i & 7);
        } else {
            return flip<NMP>(w, m, t, i);
        }
    }

    // Planar mask format: one word holds the 32 bits of ONE mask for the 32 elements a lane holds in a
    // chunk; element e of tile t (pair e/2, half e%2) has its bit here.
    __host__ __device__ static constexpr int planar_bit(int t, int e) { return 4 * t + e / 2 + 16 * (e & 1); }
    // W fragment of tile t flipped by two masks at once (ma, mb: their plane words): the two words ride
    // in one 64-bit register pair, so one 64-bit shift per register of the fragment serves both masks.
    __device__ static __forceinline__ void flip_planar2(frag w, uint32_t ma, uint32_t mb, int t, frag &ra, frag &rb)
    {
        const uint64_t mm = ((uint64_t)mb << 32) | ma;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint64_t s = shl64(mm, 15 - (4 * t + p));
            ra[p] = w[p] ^ ((uint32_t)s & 0x80008000u);
            rb[p] = w[p] ^ ((uint32_t)(s >> 32) & 0x80008000u);
        }
    }
};

struct Bf16Traits : Half16Common {
    __device__ static __forceinline__ f32x4 mma(frag a, frag b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ uint32_t to_bits(float f) { return f32_to_bf16_bits(f); }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return bf16_bits_to_f32(b); }
    __device__ static __forceinline__ void store4(void *out, long idx, f32x4 v)
    {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        *reinterpret_cast<bf16x4 *>(static_cast<uint16_t *>(out) + idx) = __builtin_convertvector(v, bf16x4);
    }
    __device__ static __forceinline__ void store1(void *out, long idx, float v)
    {
        static_cast<uint16_t *>(out)[idx] = (uint16_t)to_bits(v);
    }
};

struct F16Traits : Half16Common {
    __device__ static __forceinline__ f32x4 mma(frag a, frag b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b),
                                                      c, 0, 0, 0);
    }
    __device__ static __forceinline__ uint32_t to_bits(float f) { return f32_to_f16_bits(f); }
    __device__ static __forceinline__ float from_bits(uint32_t b) { return f16_bits_to_f32(b); }
    __device__ static __forceinline__ void store4(void *out, long idx, f32x4 v)
    {
        typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
        *reinterpret_cast<f16x4 *>(static_cast<uint16_t *>(out) + idx) = __builtin_convertvector(v, f16x4);
    }
    __device__ static __forceinline__ void store1(void *out, long idx, float v)
    {
        static_cast<uint16_t *>(out)[idx] = (uint16_t)to_bits(v);
    }
};

struct F32Traits {
    typedef f32x4 frag;                       // 4 consecutive k, one register each
    static constexpr int TILES = 8;           // 16 k per tile
    static constexpr int TILE_K = 16;
    static constexpr int LANE_K = 4;
    static constexpr int ELEM_BYTES = 4;

    __device__ static __forceinline__ f32x4 mma(frag a, frag b, f32x4 c)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], c, 0, 0, 0);
        return c;
    }

    template <int NMP>
    __device__ static __forceinline__ frag flip(frag w, const uint32_t (&m)[NMP], int t, int i)
    {
        frag r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lin = (4 * t + e) * NMP + i;
            r[e] = __uint_as_float(__float_as_uint(w[e]) ^ ((m[lin >> 5] << (31 - (lin & 31))) & 0x80000000u));
        }
        return r;
    }

    template <int NMP>
    __device__ static __forceinline__ frag flip_at(frag w, const uint32_t (&m)[NMP], int t, int i)
    {
        frag r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int lin0 = (4 * t + e) * NMP;
            r[e] = __uint_as_float(__float_as_uint(w[e]) ^ ((m[lin0 >> 5] << (31 - (lin0 & 31) - i)) & 0x80000000u));
        }
        return r;
    }

    // planar mask format (see Half16Common): element e of tile t is bit 4t + e of a mask's word
    __host__ __device__ static constexpr int planar_bit(int t, int e) { return 4 * t + e; }
    __device__ static __forceinline__ void flip_planar2(frag w, uint32_t ma, uint32_t mb, int t, frag &ra, frag &rb)
    {
        const uint64_t mm = ((uint64_t)mb << 32) | ma;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t s = shl64(mm, 31 - (4 * t + e));
            ra[e] = __uint_as_float(__float_as_uint(w[e]) ^ ((uint32_t)s & 0x80000000u));
            rb[e] = __uint_as_float(__float_as_uint(w[e]) ^ ((uint32_t)(s >> 32) & 0x80000000u));
        }
    }

    __device__ static __forceinline__ void store4(void *out, long idx, f32x4 v)
    {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(out) + idx) = v;
    }
    __device__ static __forceinline__ void store1(void *out, long idx, float v) { static_cast<float *>(out)[idx] = v; }
};

// the traits' names as they appear in a kernel instantiation's name (host side, for the plan query)
template <typename Tr> constexpr const char *traits_name();
template <> constexpr const char *traits_name<Bf16Traits>() { return "Bf16Traits"; }
template <> constexpr const char *traits_name<F16Traits>() { return "F16Traits"; }
template <> constexpr const char *traits_name<F32Traits>() { return "F32Traits"; }

// ---- what a launch computes ---------------------------------------------------------------
enum Mode {
    kModeMglu = 0,         // out = sum_i swish(gate_i) * value_i             (Eq. 3)
    kModeProjections = 1,  // t, gate_i, value_i in fp32                      (Alg. 1's z)
    kModeSwiglu = 2,       // out = swish(x Wg) * (x Wv), two weight streams  (Eq. 1)
    kModeLinear = 3,       // out = x W, no masks, no activation              (output projection W_o)
    kModeMgluVariant = 4   // out = sum_i G_i g(gate_i) * value_i with the gate function, the masked
                           // branches and the route weights chosen at run time (appendix variants);
                           // kept apart so that the main form's epilogue stays free of those choices
};

// accumulator sets a mode keeps per output tile
__host__ __device__ constexpr int sets_of(int mode, int nmp)
{
    return mode == kModeSwiglu ? 2 : mode == kModeLinear ? 1 : 1 + nmp;
}

// What the fused epilogue applies to the reduced sums (appendix of the paper):
//   gate_fn   0 Swish, 1 GELU (exact Gaussian CDF), 2 ReLU          ("Other Activation Functions")
//   mask_use  bit 0: the gate branch is dense (x W), bit 1: the value branch is dense
//             ("Partial Mask Ablation": 1 no gate mask, 2 no value mask, 3 no masks)
//   route     null, or fp32 weights G(x)_i of the Top-K routed form: mask i of token tok at
//             route[tok * route_stride + i] (the stride is the layer's mask count; n_masks here may be
//             the count of a sub-range of masks that one launch covers)
struct EpilogueParams {
    int n_masks;
    int gate_fn;
    int mask_use;
    const float *route;
    int route_stride;
};

// Sign-flip form of the complement trick (Alg. 1 writes s_i and t - s_i): with
// t = sum v and dsum_i = sum (1 - 2 M_i) v over the same terms in the same order,
//   gate_i = (t - dsum_i) / 2,   value_i = (t + dsum_i) / 2.
// An all-value mask leaves W untouched, so dsum_i = t bit for bit and gate_i = 0 exactly.
// An all-gate mask gives dsum_i = -t only up to the last bit (the matrix cores' accumulation
// is not exactly sign-symmetric), so value_i is then a few ulp of t instead of exactly 0.
__device__ __forceinline__ float gate_of(float t, float dsum) { return 0.5f * (t - dsum); }
__device__ __forceinline__ float value_of(float t, float dsum) { return 0.5f * (t + dsum); }

__device__ __forceinline__ float gate_fn_apply(int gate_fn, float z)
{
    if (gate_fn == 1) return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
    if (gate_fn == 2) return fmaxf(z, 0.0f);
    return swish(z);
}

// Route weights G(x)_i of one token (1 for every mask when the layer is not routed).  Loaded ahead
// of the K loop where the latency of this small read would otherwise sit at the end of a workgroup.
template <int NMP>
__device__ __forceinline__ void route_weights(const EpilogueParams &e, long tok, bool valid, float (&rw)[NMP])
{
#pragma unroll
    for (int i = 0; i < NMP; ++i) rw[i] = 1.0f;
    if (e.route && valid) {
#pragma unroll
        for (int i = 0; i < NMP; ++i)
            if (i < e.n_masks) rw[i] = e.route[tok * e.route_stride + i];
    }
}

// The Swish term with both halves folded in and its factor -1/4 left out:
//   swish(g) v = g v / (1 + exp(-g)),  g v = (t - dsum)(t + dsum) / 4,  exp(-g) = 2^((dsum - t) log2(e) / 2)
// -- seven instructions instead of ten.  The product is rounded on its own (never fused into the sum
// that follows), so that every epilogue, whatever it does with the term, sees the same bits; the
// factor is a power of two and may be applied to a term or to a sum of terms alike.
__device__ __forceinline__ float swish_term_x4(float t, float dsum)
{
#pragma clang fp contract(off)
    const float u = dsum - t;
    const float den = 1.0f + __builtin_amdgcn_exp2f(u * 0.72134752044448170f);
    return (u * (t + dsum)) * __builtin_amdgcn_rcpf(den);
}

// One mask's term of Eq. 3 from the reduced sums t and dsum_i (before any route weight).
__device__ __forceinline__ float mglu_term(const EpilogueParams &e, float t, float dsum)
{
    if (e.gate_fn == 0 && e.mask_use == 0) return -0.25f * swish_term_x4(t, dsum);
    const float gate = (e.mask_use & 1) ? t : gate_of(t, dsum);
    const float value = (e.mask_use & 2) ? t : value_of(t, dsum);
    return gate_fn_apply(e.gate_fn, gate) * value;
}

// One output element of the layer from its reduced sums: t and dsum[0 .. n_masks).
// PLAIN: the caller's mode fixes Swish, both masks in use and no route weights at compile time.
template <int NMP, bool PLAIN>
__device__ __forceinline__ float mglu_mix(const EpilogueParams &e, const float (&rw)[NMP], float t,
                                          const float (&dsum)[NMP])
{
    float sum = 0.f;
    if constexpr (PLAIN) {
#pragma unroll
        for (int i = 0; i < NMP; ++i) {
            if (i >= e.n_masks) break;
            const float term = swish_term_x4(t, dsum[i]);
            sum = i == 0 ? term : sum + term;
        }
        return -0.25f * sum;
    } else {
#pragma unroll
        for (int i = 0; i < NMP; ++i) {
            if (i >= e.n_masks) break;
            const float term = mglu_term(e, t, dsum[i]);
            sum += e.route ? rw[i] * term : term;
        }
        return sum;
    }
}

}  // namespace mglu
