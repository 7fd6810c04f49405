// One read of a dense bf16 matrix x producing BOTH of its MS-EDEN quantizations: Q(x), scale
// groups and rotation chunks along the rows of x, and Q(x^T), along its columns, each with its own
// rotation and rounding seeds.  The backward pass of a linear layer (paper Sec. 5) needs the output
// gradient E in both orientations (dX = Q(E) Q(W^T)^T over d_out, dW = Q(E^T) Q(X^T)^T over the
// tokens); Sec. 7 ("Fused Re-Quantization Kernel") describes the backward quantizers as fused
// kernels around a single load of their operand.  Bytes are identical to those of the two
// separate quantizer calls.
//
// A block takes one 128 x 128 tile: 16-byte loads along the rows (256 contiguous bytes per row)
// into an LDS image, then the row part in the octet layout (a lane = one 16-element group of a
// row, 4 rows per lane) and the column part in the quad layout (a lane quad = one 128-chunk of
// two columns), both reading the image.  LDS image: row r keeps its 4-byte word w (two bf16
// columns) at word w ^ (8 (r / 32)): the column part's 64 lanes (rows 32 q + i for q = 0..3,
// 16 consecutive words) then hit 32 different banks per half wave, and the row part's 32-byte
// groups stay contiguous (the xor only permutes whole groups).
#include "qii_device.h"
#include "qii_internal.h"
#include "quantize_core.h"
#include "quantize_lanes.h"

namespace qii {
namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct PairSide {
    uint32_t sign[4];      // the 128 rotation signs (host-side Philox), bit j of word j / 32
    uint64_t seed_sr;
    const float *amax;     // QII_MS_EDEN: max |rotated tensor| (device scalar)
    uint8_t *codes;
    uint8_t *scales;
    float *tensor_scale;
    float *tbuf;           // QII_MS_EDEN_PH: corrected pseudo-scales, one f32 per group
    uint32_t *amax_out;    // QII_MS_EDEN_PH: spread running maximum (nullable)
};

struct PairArgs {
    const uint16_t *x;
    int64_t ld;            // elements
    int64_t rows, cols;    // of x; both multiples of 128
    int tiles_x;           // tiles along a row of x
    PairSide r, c;         // r: Q(x), rows x cols;  c: Q(x^T), cols x rows
};

constexpr uint32_t kNoStore = 0xFFFFFFF0u;   // a lane offset beyond every buffer descriptor: the store is dropped

__device__ __forceinline__ __amdgpu_buffer_rsrc_t region(const void *base, int64_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

template <int kMode>
__global__ __launch_bounds__(256) void quantize_pair_kernel(PairArgs a)
{
    __shared__ __align__(16) uint8_t tile[128 * 256];
    __shared__ float inv_r[128], inv_c[128];
    __shared__ float wave_m[2][4];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int ty = (int)blockIdx.x / a.tiles_x, tx = (int)blockIdx.x - ty * a.tiles_x;
    const int64_t row0 = (int64_t)ty * 128, col0 = (int64_t)tx * 128;

    // ---- the tile's loads first: 8 pieces of 16 bytes per thread, 16 threads per row
    u32x4 w[8];
    {
        const __amdgpu_buffer_rsrc_t src = region(a.x + row0 * a.ld + col0, (127 * a.ld + 128) * 2);
        const uint32_t voff = (uint32_t)(((t >> 4) * a.ld + (t & 15) * 8) * 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = __builtin_amdgcn_raw_buffer_load_b128(src, voff, (int)(i * 16 * a.ld * 2), 0);
    }

    // ---- tensor constants and reciprocal tables of the two sides while the loads are in flight
    TensorConsts tcr = TensorConsts{}, tcc = TensorConsts{};
    if (kMode == QII_MS_EDEN) {
        tcr = tensor_consts(QII_MS_EDEN, *a.r.amax);
        tcc = tensor_consts(QII_MS_EDEN, *a.c.amax);
        if (blockIdx.x == 0 && t == 0) {
            *a.r.tensor_scale = tcr.x32;
            *a.c.tensor_scale = tcc.x32;
        }
        const uint32_t b = t & 127;
        const float x32 = t < 128 ? tcr.x32 : tcc.x32;
        (t < 128 ? inv_r : inv_c)[b] = b == 0u ? 0.0f : 1.0f / (e4m3_decode(b) * x32);
    }

    // ---- LDS image (swizzled, see the file header)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = (t >> 4) + 16 * i, p = (t & 15) ^ (2 * (r >> 5));
        *reinterpret_cast<u32x4 *>(tile + r * 256 + p * 16) = w[i];
    }
    __syncthreads();

    float m_r = 0.0f, m_c = 0.0f;

    // ---- row part: Q(x).  quad = 4 consecutive rows of the tile (one draw call serves them);
    // the 8 lanes of an octet own the 8 groups of those rows inside the tile
    {
        const OctetLane L = octet_lane(lane, a.r.sign);
        uint32_t mask[8];
        make_masks<true>(L.sign16, mask);
        const int quad = 8 * wave + (lane >> 3);
        const int64_t G = a.cols / 16, cpitch = a.cols / 2;
        uint32_t draw[4] = {0u, 0u, 0u, 0u};
        if (kMode == QII_MS_EDEN) {
            const U4 d = philox_seeded(a.r.seed_sr, (uint32_t)(tx * 8 + L.blk), (uint32_t)(ty * 32 + quad), 0, kStreamScale);
            draw[0] = d.x >> 12; draw[1] = d.y >> 12; draw[2] = d.z >> 12; draw[3] = d.w >> 12;
        }
        // this tile's part of the outputs: 64 code bytes, 8 scale bytes (or 8 f32) per row
        const __amdgpu_buffer_rsrc_t rc = region(a.r.codes + row0 * cpitch + col0 / 2, 127 * cpitch + 64);
        const __amdgpu_buffer_rsrc_t rs = region(a.r.scales + row0 * G + col0 / 16, 127 * G + 8);
        const bool zero = kMode == QII_MS_EDEN && tcr.zero;   // uniform: an all-zero tensor is emitted as zero bytes
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = 4 * quad + it;   // (r / 32 == wave)
            const uint8_t *src = tile + r * 256 + ((L.blk ^ wave) * 32);
            const u32x4 q0 = *reinterpret_cast<const u32x4 *>(src), q1 = *reinterpret_cast<const u32x4 *>(src + 16);
            const uint32_t w8[8] = {q0[0], q0[1], q0[2], q0[3], q1[0], q1[1], q1[2], q1[3]};
            float v[16];
            unpack_bf16x16<true>(w8, v, mask);
            rht128_lane(v, L);
            uint32_t packed[2];
            const uint32_t vc = (uint32_t)(r * cpitch) + 8u * L.blk;
            if (kMode == QII_MS_EDEN_PH) {
                float gmax;
                const float tt = posthoc_group16(v, packed, gmax);
                __builtin_amdgcn_raw_buffer_store_b64(u32x2{packed[0], packed[1]}, rc, vc, 0, 0);
                a.r.tbuf[(row0 + r) * G + col0 / 16 + L.blk] = tt;
                m_r = fmaxf(m_r, gmax);
                continue;
            }
            uint32_t b = quantize_group16<QII_MS_EDEN, -1, true>(v, tcr, draw[it], a.r.seed_sr, row0 + r, tx * 8 + L.blk, packed, inv_r);
            if (zero) { packed[0] = 0u; packed[1] = 0u; b = 0u; }
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{packed[0], packed[1]}, rc, vc, 0, 0);
            const uint2 sc = gather_scale_bytes(b, L.blk);
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{sc.x, sc.y}, rs, L.blk == 0 ? (uint32_t)(r * G) : kNoStore, 0, 0);
        }
    }

    // ---- column part: Q(x^T).  The tile is chunk `ty` of the columns' 128-chunks; wave w takes the
    // tile's columns 32 w .. 32 w + 31, a lane quad two of them, lane q of the quad rows 32 q .. 32 q + 31
    {
        const int q = lane & 3, jp = lane >> 2;
        const uint8_t *src = tile + (32 * q) * 256 + 4 * ((16 * wave + jp) ^ (8 * q));
        uint32_t raw[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) raw[i] = *reinterpret_cast<const uint32_t *>(src + i * 256);
        const uint32_t sw = q == 0 ? a.c.sign[0] : q == 1 ? a.c.sign[1] : q == 2 ? a.c.sign[2] : a.c.sign[3];
        float v[2][32];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const uint32_t flip = ((sw >> i) & 1u) << 31;
            v[0][i] = u2f((raw[i] << 16) ^ flip);
            v[1][i] = u2f((raw[i] & 0xFFFF0000u) ^ flip);
        }
        fwht128_quad(v[0], q);
        fwht128_quad(v[1], q);
        const int64_t chunk = ty, j0 = col0 + 32 * wave + 2 * jp;
        const int64_t G = a.rows / 16, cpitch = a.rows / 2;
        uint32_t draw[2][2] = {{0u, 0u}, {0u, 0u}};
        if (kMode == QII_MS_EDEN) octet_draws(draw, a.c.seed_sr, chunk, j0, q);
        const bool zero = kMode == QII_MS_EDEN && tcc.zero;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            uint32_t codes[4];
            if (kMode == QII_MS_EDEN_PH) {
                float tt[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float gmax;
                    tt[h] = posthoc_group16(v[e] + 16 * h, codes + 2 * h, gmax);
                    m_c = fmaxf(m_c, gmax);
                }
                *reinterpret_cast<uint4 *>(a.c.codes + (j0 + e) * cpitch + chunk * 64 + 16 * q) = make_uint4(codes[0], codes[1], codes[2], codes[3]);
                *reinterpret_cast<float2 *>(a.c.tbuf + (j0 + e) * G + chunk * 8 + 2 * q) = make_float2(tt[0], tt[1]);
                continue;
            }
            uint32_t sc = 0u;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t b = quantize_group16<QII_MS_EDEN, -1, true>(v[e] + 16 * h, tcc, draw[e][h], a.c.seed_sr, j0 + e,
                                                                           chunk * 8 + 2 * q + h, codes + 2 * h, inv_c);
                sc |= b << (8 * h);
            }
            if (zero) { codes[0] = codes[1] = codes[2] = codes[3] = 0u; sc = 0u; }
            const uint2 s8 = gather_quad_scales(sc, q);
            *reinterpret_cast<uint4 *>(a.c.codes + (j0 + e) * cpitch + chunk * 64 + 16 * q) = make_uint4(codes[0], codes[1], codes[2], codes[3]);
            if (q == 0) *reinterpret_cast<uint2 *>(a.c.scales + (j0 + e) * G + chunk * 8) = s8;
        }
    }

    // ---- post hoc scheme: the block's two maxima into the spread running maxima
    if (kMode == QII_MS_EDEN_PH && (a.r.amax_out || a.c.amax_out)) {   // uniform
        m_r = wave_max(m_r);
        m_c = wave_max(m_c);
        if (lane == 0) { wave_m[0][wave] = m_r; wave_m[1][wave] = m_c; }
        __syncthreads();
        if (t < 2) {
            uint32_t *out = t == 0 ? a.r.amax_out : a.c.amax_out;
            if (out) max_to_global(fmaxf(fmaxf(wave_m[t][0], wave_m[t][1]), fmaxf(wave_m[t][2], wave_m[t][3])),
                                   amax_spread_word(out, blockIdx.x));
        }
    }
}

}  // namespace

// dense bf16, no transposition, both dimensions multiples of 128, 16-byte aligned rows, and
// offsets inside a tile's rows that fit the 32-bit fields of a buffer descriptor
bool pair_kernel_applies(const Source &src, int64_t rows, int64_t cols)
{
    return src.kind == kSrcBF16 && !src.transpose && rows > 0 && cols > 0 && rows % 128 == 0 && cols % 128 == 0 &&
           src.ld % 8 == 0 && (reinterpret_cast<uintptr_t>(src.x) & 15) == 0 && src.ld <= ((int64_t)1 << 21) &&
           cols <= ((int64_t)1 << 23) && rows <= ((int64_t)1 << 23) && (rows / 128) * (cols / 128) < ((int64_t)1 << 31);
}

hipError_t launch_quantize_pair(const PairQuantizeArgs &p, hipStream_t s)
{
    PairArgs a;
    a.x = reinterpret_cast<const uint16_t *>(p.src.x);
    a.ld = p.src.ld; a.rows = p.rows; a.cols = p.cols;
    a.tiles_x = (int)(p.cols / 128);
    const PairQuantizeArgs::Side *in[2] = {&p.r, &p.c};
    PairSide *out[2] = {&a.r, &a.c};
    for (int i = 0; i < 2; ++i) {
        const U4 w = philox_seeded(in[i]->seed_rht, 0, 0, 0, kStreamRht);
        out[i]->sign[0] = w.x; out[i]->sign[1] = w.y; out[i]->sign[2] = w.z; out[i]->sign[3] = w.w;
        out[i]->seed_sr = in[i]->seed_sr;
        out[i]->amax = in[i]->amax;
        out[i]->codes = in[i]->codes; out[i]->scales = in[i]->scales; out[i]->tensor_scale = in[i]->tensor_scale;
        out[i]->tbuf = in[i]->tbuf; out[i]->amax_out = in[i]->amax_accum;
    }
    const dim3 grid((unsigned)((p.rows / 128) * (p.cols / 128))), block(256);
    if (p.mode == QII_MS_EDEN_PH) hipLaunchKernelGGL((quantize_pair_kernel<QII_MS_EDEN_PH>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((quantize_pair_kernel<QII_MS_EDEN>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace qii
