// Weight compressor, decompressor and dense-twin packer (Fig. 1; Sec. 3.1 Eq. 2; Sec. 3.3 Eq. 6).
// Integer / bit work only: no floating-point instruction touches a weight.
#include "ss_internal.h"

namespace ss {

// ---------------------------------------------------------------------------------------------
// header
// ---------------------------------------------------------------------------------------------
__global__ void write_header_kernel(uint32_t *hdr, uint32_t magic, int cout, int cin, int kh, int kw,
                                    int dtype, int korder, int Mt, int Ks)
{
    int i = threadIdx.x;            // 64 threads, one word each
    uint32_t v = 0;
    switch (i) {
        case 0: v = magic; break;
        case 1: v = 1; break;
        case 2: v = (uint32_t)cout; break;
        case 3: v = (uint32_t)cin; break;
        case 4: v = (uint32_t)kh; break;
        case 5: v = (uint32_t)kw; break;
        case 6: v = (uint32_t)dtype; break;
        case 7: v = (uint32_t)korder; break;
        case 8: v = (uint32_t)Mt; break;
        case 9: v = (uint32_t)Ks; break;
        case 10: v = kNoBadBlock; break;
        default: break;
    }
    hdr[i] = v;
}

// ---------------------------------------------------------------------------------------------
// compressor
//
// One thread produces one lane of one value tile: 8 packed values (16 bytes) and the 16 index
// bits that go with them.  Lane l of tile (mt, ks) owns row 32*mt + l%32 and the four blocks
// 8*ks + {0,1,4,5} + 2*(l/32) of that row, i.e. the reduction indices 32*ks + 8*(l/32) + [0,8)
// and 32*ks + 16 + 8*(l/32) + [0,8): this is where gfx950's 32x32x32 sparse MFMA expects the
// A operand of a lane to come from, given that lane l of the B operand holds the 16 consecutive
// reduction indices 32*ks + 16*(l/32) + [0,16).
// ---------------------------------------------------------------------------------------------
// binary32 sum of two 16-bit values, rounded to nearest even back to the storage type
template <int DT>
__device__ __forceinline__ uint32_t add16(uint32_t a, uint32_t b)
{
    if constexpr (DT == SS_F16) {
        float s = (float)__builtin_bit_cast(_Float16, (uint16_t)a) + (float)__builtin_bit_cast(_Float16, (uint16_t)b);
        return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)s);
    } else {
        float s = __builtin_bit_cast(float, a << 16) + __builtin_bit_cast(float, b << 16);
        return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)s);
    }
}

// UPD: the weights are first moved to V = W + U (written back over W; every element belongs to exactly one
// thread's blocks), then V is packed.
template <int DT, bool UPD>
__global__ __launch_bounds__(256) void compress_kernel(uint16_t *__restrict__ W, const uint16_t *__restrict__ U,
                                                       const uint8_t *__restrict__ M, uint8_t *__restrict__ packed,
                                                       int cout, int K, int Mt, int Ks, int Kp)
{
    int tid = blockIdx.x * 256 + threadIdx.x;
    int total = Mt * Ks * 64;
    if (tid >= total) return;
    int lane = tid & 63;
    int tile = tid >> 6;
    int ks = tile % Ks;
    int mt = tile / Ks;
    int row = mt * 32 + (lane & 31);
    int ga = lane >> 5;
    int G = K >> 2;

    uint32_t v[4];
    uint32_t nibbles = 0;
    uint32_t *first_bad = reinterpret_cast<uint32_t *>(packed) + kHdrFirstBad;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        int g = 8 * ks + 4 * (j >> 1) + 2 * ga + (j & 1);
        uint32_t pair = 0, nib = 0x4;
        if (row < cout && g < G) {
            size_t e = (size_t)row * K + 4 * (size_t)g;
            uint32_t m = *reinterpret_cast<const uint32_t *>(M + e);
            uint2 w = *reinterpret_cast<const uint2 *>(W + e);
            if constexpr (UPD) {
                const uint2 u = *reinterpret_cast<const uint2 *>(U + e);
                w.x = add16<DT>(w.x & 0xFFFFu, u.x & 0xFFFFu) | (add16<DT>(w.x >> 16, u.x >> 16) << 16);
                w.y = add16<DT>(w.y & 0xFFFFu, u.y & 0xFFFFu) | (add16<DT>(w.y >> 16, u.y >> 16) << 16);
                *reinterpret_cast<uint2 *>(W + e) = w;
            }
            bool ok = ((m & 0xFEFEFEFEu) == 0) && (__popc(m) == 2);
            if (ok) {
                int i0 = (__ffs(m) - 1) >> 3;
                int i1 = (31 - __clz(m)) >> 3;
                uint64_t w64 = ((uint64_t)w.y << 32) | w.x;
                uint32_t v0 = (uint32_t)(w64 >> (16 * i0)) & 0xFFFFu;
                uint32_t v1 = (uint32_t)(w64 >> (16 * i1)) & 0xFFFFu;
                pair = v0 | (v1 << 16);
                nib = (uint32_t)(i0 | (i1 << 2));
            } else {
                atomicMin(first_bad, (uint32_t)((size_t)row * G + g));
            }
        }
        v[j] = pair;
        nibbles |= nib << (4 * j);
    }
    uint4 out = make_uint4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<uint4 *>(packed + kHeaderBytes + ((size_t)tile * 64 + lane) * 16) = out;
    uint16_t *meta = reinterpret_cast<uint16_t *>(packed + kHeaderBytes + (size_t)Mt * Ks * 1024);
    size_t mi = (((size_t)mt * Kp + (ks >> 1)) * 64 + lane) * 2 + (ks & 1);
    meta[mi] = (uint16_t)nibbles;
    if ((Ks & 1) && ks == Ks - 1) meta[mi + 1] = 0x4444;   // unused upper half of the last pair
}

// thread per (row, block): inverse permutation, writes 4 elements (8 bytes)
__global__ __launch_bounds__(256) void decompress_kernel(const uint8_t *__restrict__ packed, uint16_t *__restrict__ Wm,
                                                         int cout, int K, int Mt, int Ks, int Kp)
{
    int G = K >> 2;
    int tid = blockIdx.x * 256 + threadIdx.x;
    if (tid >= cout * G) return;
    int g = tid % G, row = tid / G;
    int mt = row >> 5, i = row & 31;
    int ks = g >> 3, gl = g & 7;
    int ga = (gl >> 1) & 1;
    int j = 2 * (gl >> 2) + (gl & 1);
    int lane = 32 * ga + i;
    const uint32_t *vals = reinterpret_cast<const uint32_t *>(packed + kHeaderBytes);
    uint32_t pair = vals[(((size_t)mt * Ks + ks) * 64 + lane) * 4 + j];
    const uint32_t *meta = reinterpret_cast<const uint32_t *>(packed + kHeaderBytes + (size_t)Mt * Ks * 1024);
    uint32_t word = meta[((size_t)mt * Kp + (ks >> 1)) * 64 + lane] >> (16 * (ks & 1));
    uint32_t nib = (word >> (4 * j)) & 0xFu;
    int i0 = nib & 3, i1 = (nib >> 2) & 3;
    uint64_t w64 = 0;
    w64 |= (uint64_t)(pair & 0xFFFFu) << (16 * i0);
    w64 |= (uint64_t)(pair >> 16) << (16 * i1);
    *reinterpret_cast<uint2 *>(Wm + (size_t)row * K + 4 * (size_t)g) = make_uint2((uint32_t)w64, (uint32_t)(w64 >> 32));
}

// Dense twin operand: thread per (tile (mt, ks, h), lane); 8 elements k = 32*ks + 16*(l/32) + 8*h + s.
__global__ __launch_bounds__(256) void dense_pack_kernel(const uint16_t *__restrict__ W, const uint8_t *__restrict__ M,
                                                         uint8_t *__restrict__ dense, int cout, int K, int Mt, int Ks)
{
    int tid = blockIdx.x * 256 + threadIdx.x;
    int total = Mt * Ks * 2 * 64;
    if (tid >= total) return;
    int lane = tid & 63;
    int tile = tid >> 6;
    int h = tile & 1;
    int ks = (tile >> 1) % Ks;
    int mt = (tile >> 1) / Ks;
    int row = mt * 32 + (lane & 31);
    int kbase = 32 * ks + 16 * (lane >> 5) + 8 * h;
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 8; s++) {
        int k = kbase + s;
        uint32_t val = 0;
        if (row < cout && k < K) {
            size_t e = (size_t)row * K + k;
            bool keep = (M == nullptr) || (M[e] != 0);
            val = keep ? (uint32_t)W[e] : 0u;
        }
        o[s >> 1] |= val << (16 * (s & 1));
    }
    *reinterpret_cast<uint4 *>(dense + kHeaderBytes + ((size_t)tile * 64 + lane) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
}

// ---------------------------------------------------------------------------------------------
// 8-bit operands (integer or FP8: bytes are copied, never interpreted).  One thread produces one lane of one value tile: 16 packed bytes and the 32 index
// bits that go with them.  Lane l of tile (mt, ks) owns row 32*mt + l%32 and, in slots 2j, 2j+1 (j = 0..7),
// block 16*ks + 8*(j/4) + 4*(l/32) + j%4: gfx950's 32x32x64 8-bit sparse MFMAs pair slot s of lane l with the
// bytes 16*(l/32) + 4*((s%8)/2) + [0,4) of the B lane of the same column in lane group s/8, and B lane groups
// hold the reduction indices 64*ks + 32*group + [0,32).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compress8_kernel(const uint8_t *__restrict__ W, const uint8_t *__restrict__ M,
                                                        uint8_t *__restrict__ packed, int cout, int K, int Mt, int Ks)
{
    int tid = blockIdx.x * 256 + threadIdx.x;
    int total = Mt * Ks * 64;
    if (tid >= total) return;
    int lane = tid & 63;
    int tile = tid >> 6;
    int ks = tile % Ks;
    int mt = tile / Ks;
    int row = mt * 32 + (lane & 31);
    int ga = lane >> 5;
    int G = K >> 2;

    uint32_t v[4] = {0, 0, 0, 0};
    uint32_t nibbles = 0;
    uint32_t *first_bad = reinterpret_cast<uint32_t *>(packed) + kHdrFirstBad;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int g = 16 * ks + 8 * (j >> 2) + 4 * ga + (j & 3);
        uint32_t pair = 0, nib = 0x4;
        if (row < cout && g < G) {
            size_t e = (size_t)row * K + 4 * (size_t)g;
            uint32_t m = *reinterpret_cast<const uint32_t *>(M + e);
            uint32_t w = *reinterpret_cast<const uint32_t *>(W + e);
            bool ok = ((m & 0xFEFEFEFEu) == 0) && (__popc(m) == 2);
            if (ok) {
                int i0 = (__ffs(m) - 1) >> 3;
                int i1 = (31 - __clz(m)) >> 3;
                pair = ((w >> (8 * i0)) & 0xFFu) | (((w >> (8 * i1)) & 0xFFu) << 8);
                nib = (uint32_t)(i0 | (i1 << 2));
            } else {
                atomicMin(first_bad, (uint32_t)((size_t)row * G + g));
            }
        }
        v[j >> 1] |= pair << (16 * (j & 1));
        nibbles |= nib << (4 * j);
    }
    *reinterpret_cast<uint4 *>(packed + kHeaderBytes + ((size_t)tile * 64 + lane) * 16) = make_uint4(v[0], v[1], v[2], v[3]);
    uint32_t *meta = reinterpret_cast<uint32_t *>(packed + kHeaderBytes + (size_t)Mt * Ks * 1024);
    meta[(size_t)tile * 64 + lane] = nibbles;
}

// thread per (row, block): inverse permutation, writes 4 bytes
__global__ __launch_bounds__(256) void decompress8_kernel(const uint8_t *__restrict__ packed, uint8_t *__restrict__ Wm,
                                                          int cout, int K, int Mt, int Ks)
{
    int G = K >> 2;
    int tid = blockIdx.x * 256 + threadIdx.x;
    if (tid >= cout * G) return;
    int g = tid % G, row = tid / G;
    int mt = row >> 5, i = row & 31;
    int ks = g >> 4, gl = g & 15;
    int ga = (gl >> 2) & 1;
    int j = 4 * (gl >> 3) + (gl & 3);
    int lane = 32 * ga + i;
    const uint16_t *vals = reinterpret_cast<const uint16_t *>(packed + kHeaderBytes);
    uint32_t pair = vals[(((size_t)mt * Ks + ks) * 64 + lane) * 8 + j];
    const uint32_t *meta = reinterpret_cast<const uint32_t *>(packed + kHeaderBytes + (size_t)Mt * Ks * 1024);
    uint32_t nib = (meta[((size_t)mt * Ks + ks) * 64 + lane] >> (4 * j)) & 0xFu;
    int i0 = nib & 3, i1 = (nib >> 2) & 3;
    uint32_t w = ((pair & 0xFFu) << (8 * i0)) | ((pair >> 8) << (8 * i1));
    *reinterpret_cast<uint32_t *>(Wm + (size_t)row * K + 4 * (size_t)g) = w;
}

// Dense twin operand: thread per (tile (mt, ks, h), lane); 16 bytes k = 64*ks + 32*(l/32) + 16*h + s.
__global__ __launch_bounds__(256) void dense_pack8_kernel(const uint8_t *__restrict__ W, const uint8_t *__restrict__ M,
                                                          uint8_t *__restrict__ dense, int cout, int K, int Mt, int Ks)
{
    int tid = blockIdx.x * 256 + threadIdx.x;
    int total = Mt * Ks * 2 * 64;
    if (tid >= total) return;
    int lane = tid & 63;
    int tile = tid >> 6;
    int h = tile & 1;
    int ks = (tile >> 1) % Ks;
    int mt = (tile >> 1) / Ks;
    int row = mt * 32 + (lane & 31);
    int kbase = 64 * ks + 32 * (lane >> 5) + 16 * h;
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 16; s++) {
        int k = kbase + s;
        uint32_t val = 0;
        if (row < cout && k < K) {
            size_t e = (size_t)row * K + k;
            bool keep = (M == nullptr) || (M[e] != 0);
            val = keep ? (uint32_t)W[e] : 0u;
        }
        o[s >> 2] |= val << (8 * (s & 3));
    }
    *reinterpret_cast<uint4 *>(dense + kHeaderBytes + ((size_t)tile * 64 + lane) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
}

}  // namespace ss

using namespace ss;

extern "C" const char *ss_status_string(int status)
{
    switch (status) {
        case SS_OK: return "SS_OK";
        case SS_ERR_INVALID_ARG: return "SS_ERR_INVALID_ARG: null pointer, bad size or unknown enum";
        case SS_ERR_BAD_MASK: return "SS_ERR_BAD_MASK: a block of 4 mask entries does not hold exactly two ones";
        case SS_ERR_UNSUPPORTED: return "SS_ERR_UNSUPPORTED: K is not a multiple of 4, or sizes exceed the index range";
        case SS_ERR_WORKSPACE: return "SS_ERR_WORKSPACE: workspace too small";
        case SS_ERR_HIP: return "SS_ERR_HIP: a HIP runtime call failed";
        default: return "unknown status";
    }
}

extern "C" int ss_packed_bytes(const ss_weight_desc *desc, size_t *packed_bytes)
{
    if (!packed_bytes) return SS_ERR_INVALID_ARG;
    int st = check_desc(desc, true);
    if (st != SS_OK) return st;
    *packed_bytes = packed_size(tile_dims(desc));
    return SS_OK;
}

extern "C" int ss_dense_bytes(const ss_weight_desc *desc, size_t *dense_bytes)
{
    if (!dense_bytes) return SS_ERR_INVALID_ARG;
    int st = check_desc(desc, false);
    if (st != SS_OK) return st;
    *dense_bytes = dense_size(tile_dims(desc));
    return SS_OK;
}

static int compress_entry(const ss_weight_desc *desc, void *W, const void *U, const uint8_t *M, void *packed,
                          int32_t *bad_row_group, void *stream)
{
    int st = check_desc(desc, true);
    if (st != SS_OK) return st;
    if (!W || !M || !packed) return SS_ERR_INVALID_ARG;
    const bool i8 = is_byte_type(desc->dtype);
    if (i8 && U) return SS_ERR_UNSUPPORTED;       // the update is defined on the 16-bit floats only
    if (!aligned(W, i8 ? 4 : 8) || !aligned(M, 4) || !aligned(packed, 16) || (U && !aligned(U, 8))) return SS_ERR_INVALID_ARG;
    TileDims t = tile_dims(desc);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(packed);
    write_header_kernel<<<1, 64, 0, s>>>(reinterpret_cast<uint32_t *>(p), kMagicSparse, desc->cout, desc->cin,
                                         desc->kh, desc->kw, desc->dtype, desc->korder, t.Mt, t.Ks);
    int total = t.Mt * t.Ks * 64;
    dim3 grid((total + 255) / 256), block(256);
    uint16_t *w = static_cast<uint16_t *>(W);
    const uint16_t *u = static_cast<const uint16_t *>(U);
    if (i8)
        compress8_kernel<<<grid, block, 0, s>>>(static_cast<const uint8_t *>(W), M, p, desc->cout, t.K, t.Mt, t.Ks);
    else if (!U)
        compress_kernel<SS_F16, false><<<grid, block, 0, s>>>(w, nullptr, M, p, desc->cout, t.K, t.Mt, t.Ks, t.Kp);
    else if (desc->dtype == SS_F16)
        compress_kernel<SS_F16, true><<<grid, block, 0, s>>>(w, u, M, p, desc->cout, t.K, t.Mt, t.Ks, t.Kp);
    else
        compress_kernel<SS_BF16, true><<<grid, block, 0, s>>>(w, u, M, p, desc->cout, t.K, t.Mt, t.Ks, t.Kp);
    if (hipGetLastError() != hipSuccess) return SS_ERR_HIP;
    uint32_t first_bad = 0;
    if (hipMemcpyAsync(&first_bad, p + 4 * kHdrFirstBad, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return SS_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SS_ERR_HIP;
    if (first_bad != kNoBadBlock) {
        if (bad_row_group) {
            bad_row_group[0] = (int32_t)(first_bad / (uint32_t)t.G);
            bad_row_group[1] = (int32_t)(first_bad % (uint32_t)t.G);
        }
        return SS_ERR_BAD_MASK;
    }
    return SS_OK;
}

extern "C" int ss_mask_compress(const ss_weight_desc *desc, const void *W, const uint8_t *M, void *packed,
                                int32_t *bad_row_group, void *stream)
{
    return compress_entry(desc, const_cast<void *>(W), nullptr, M, packed, bad_row_group, stream);   // W is only read
}

extern "C" int ss_mask_update_compress(const ss_weight_desc *desc, void *W, const void *U, const uint8_t *M,
                                       void *packed, int32_t *bad_row_group, void *stream)
{
    if (!U) return SS_ERR_INVALID_ARG;
    return compress_entry(desc, W, U, M, packed, bad_row_group, stream);
}

extern "C" int ss_mask_decompress(const ss_weight_desc *desc, const void *packed, void *W_masked_out, void *stream)
{
    int st = check_desc(desc, true);
    if (st != SS_OK) return st;
    if (!packed || !W_masked_out) return SS_ERR_INVALID_ARG;
    const bool i8 = is_byte_type(desc->dtype);
    if (!aligned(packed, 16) || !aligned(W_masked_out, i8 ? 4 : 8)) return SS_ERR_INVALID_ARG;
    TileDims t = tile_dims(desc);
    int total = desc->cout * t.G;
    if (i8) {
        decompress8_kernel<<<(total + 255) / 256, 256, 0, static_cast<hipStream_t>(stream)>>>(
            static_cast<const uint8_t *>(packed), static_cast<uint8_t *>(W_masked_out), desc->cout, t.K, t.Mt, t.Ks);
        return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
    }
    decompress_kernel<<<(total + 255) / 256, 256, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const uint8_t *>(packed), static_cast<uint16_t *>(W_masked_out), desc->cout, t.K, t.Mt, t.Ks, t.Kp);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}

extern "C" int ss_weights_check(const ss_weight_desc *desc, const void *weights, int32_t sparse, void *stream)
{
    int st = check_desc(desc, sparse != 0);
    if (st != SS_OK) return st;
    if (!weights || !aligned(weights, 16)) return SS_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t hdr[kHdrFirstBad + 1];
    if (hipMemcpyAsync(hdr, weights, sizeof(hdr), hipMemcpyDeviceToHost, s) != hipSuccess) return SS_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SS_ERR_HIP;
    const TileDims t = tile_dims(desc);
    const uint32_t want[10] = {sparse ? kMagicSparse : kMagicDense, 1u, (uint32_t)desc->cout, (uint32_t)desc->cin,
                               (uint32_t)desc->kh, (uint32_t)desc->kw, (uint32_t)desc->dtype, (uint32_t)desc->korder,
                               (uint32_t)t.Mt, (uint32_t)t.Ks};
    for (int i = 0; i < 10; i++)
        if (hdr[i] != want[i]) return SS_ERR_INVALID_ARG;
    if (sparse && hdr[kHdrFirstBad] != kNoBadBlock) return SS_ERR_BAD_MASK;
    return SS_OK;
}

extern "C" int ss_dense_pack(const ss_weight_desc *desc, const void *W, const uint8_t *M, void *dense, void *stream)
{
    int st = check_desc(desc, false);
    if (st != SS_OK) return st;
    if (!W || !dense) return SS_ERR_INVALID_ARG;
    if (!aligned(W, is_byte_type(desc->dtype) ? 1 : 2) || !aligned(dense, 16)) return SS_ERR_INVALID_ARG;
    TileDims t = tile_dims(desc);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *p = static_cast<uint8_t *>(dense);
    write_header_kernel<<<1, 64, 0, s>>>(reinterpret_cast<uint32_t *>(p), kMagicDense, desc->cout, desc->cin,
                                         desc->kh, desc->kw, desc->dtype, desc->korder, t.Mt, t.Ks);
    int total = t.Mt * t.Ks * 2 * 64;
    if (is_byte_type(desc->dtype))
        dense_pack8_kernel<<<(total + 255) / 256, 256, 0, s>>>(static_cast<const uint8_t *>(W), M, p, desc->cout, t.K,
                                                               t.Mt, t.Ks);
    else
        dense_pack_kernel<<<(total + 255) / 256, 256, 0, s>>>(static_cast<const uint16_t *>(W), M, p, desc->cout, t.K,
                                                              t.Mt, t.Ks);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_HIP;
}
