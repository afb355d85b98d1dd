// Internal declarations shared by the HIP translation units of the library (not installed).
#ifndef SS_INTERNAL_H_
#define SS_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/ss.h"

namespace ss {

constexpr uint32_t kMagicSparse = 0x34325353u;   // "SS24"
constexpr uint32_t kMagicDense  = 0x44325353u;   // "SS2D"
constexpr uint32_t kNoBadBlock  = 0xFFFFFFFFu;
constexpr int kHeaderBytes = 256;                // 64 x uint32
constexpr int kHdrFirstBad = 10;                 // word index of the first-invalid-block field

// Tile counts of a weight matrix [cout][K]: 32-row tiles, reduction steps (32 16-bit elements or 64 bytes), index tiles.
struct TileDims {
    int K, G, Mt, Ks, Kp;
};

inline TileDims tile_dims(const ss_weight_desc *d)
{
    TileDims t;
    t.K = d->cin * d->kh * d->kw;
    t.G = t.K / 4;
    t.Mt = (d->cout + 31) / 32;
    if (d->dtype == SS_I8 || d->dtype == SS_F8) {          // reduction steps of 64 bytes, one index word per step
        t.Ks = (t.K + 63) / 64;
        t.Kp = t.Ks;
    } else {
        t.Ks = (t.K + 31) / 32;
        t.Kp = (t.Ks + 1) / 2;
    }
    return t;
}

// Validates the descriptor.  `need_groups`: the sparse representation needs K % 4 == 0.
inline int check_desc(const ss_weight_desc *d, bool need_groups)
{
    if (!d) return SS_ERR_INVALID_ARG;
    if (d->cout <= 0 || d->cin <= 0 || d->kh <= 0 || d->kw <= 0) return SS_ERR_INVALID_ARG;
    if (d->dtype != SS_F16 && d->dtype != SS_BF16 && d->dtype != SS_I8 && d->dtype != SS_F8) return SS_ERR_INVALID_ARG;
    if (d->korder != SS_K_CRS && d->korder != SS_K_RSC) return SS_ERR_INVALID_ARG;
    int64_t K = (int64_t)d->cin * d->kh * d->kw;
    if (K > (1 << 24) || (int64_t)d->cout * ((K + 63) / 64 * 64) >= (1ll << 31)) return SS_ERR_UNSUPPORTED;
    if (need_groups && (K % 4) != 0) return SS_ERR_UNSUPPORTED;
    return SS_OK;
}

inline size_t packed_size(const TileDims &t)
{
    return (size_t)kHeaderBytes + (size_t)t.Mt * t.Ks * 1024 + (size_t)t.Mt * t.Kp * 256;
}
inline size_t dense_size(const TileDims &t)
{
    return (size_t)kHeaderBytes + (size_t)t.Mt * t.Ks * 2048;
}

constexpr bool is_byte_type(int dtype) { return dtype == SS_I8 || dtype == SS_F8; }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace ss

#endif
