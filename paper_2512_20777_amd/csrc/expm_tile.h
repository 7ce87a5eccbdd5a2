// Staging geometry shared by the product kernels (square rounds and rectangular low-rank products), gfx950.
//
// A workgroup of 256 threads (2 x 2 waves) owns a (32 WT) x (32 WT) output tile and walks the inner dimension in
// k-blocks of 128 bytes per left row (16 fp64 / 32 fp32).  One staged k-block is a left tile of 32 WT rows x 8
// sixteen-byte vectors followed by a right tile of BK rows x (32 WT) elements; each thread moves WT vectors of either.
//
//   register staging: left rows are padded to 144 bytes, and each 16-lane group of a wave owns a contiguous run of
//       k inside the k-block, so a left fragment is two conflict-free 16-byte reads; right rows are rotated by 16
//       elements per k-group (row / KQ) instead of padded, so the four groups of a fragment read hit different banks.
//   straight into LDS (global_load_lds, 16 bytes per lane, lane l of a wave lands at a wave-uniform base + 16 l):
//       a tile has to be a sequence of 16-byte slots in lane order, so the left tile is unpadded (128-byte rows) and
//       swizzled -- slot (row, v') holds k-vector v' ^ ((row / 2) & 7) -- and the rotation of the right tile is
//       applied on the global side: the lane that owns slot (row, v') fetches column vector v' - rot(row).
//
// Both layouts are read back with the same fragment offsets (left_read / right_read_base).
#pragma once

#include <hip/hip_runtime.h>

namespace expmk {

constexpr int kTileThreads = 256;
constexpr int kLeftPitchPadded = 144;   // bytes per left row in LDS with register staging: 128 data + 16 pad

template <typename T> struct Tile;
template <> struct Tile<double> {
    static constexpr int BK = 16;        // k-block: 128 bytes of a row
    static constexpr int VN = 2;         // elements per 16-byte vector
    using vec_t = double2;
};
template <> struct Tile<float> {
    static constexpr int BK = 32;
    static constexpr int VN = 4;
    using vec_t = float4;
};

// bytes of one staged k-block (left tile, then right tile)
template <typename T, int WT> constexpr int stage_bytes(bool dma = false)
{
    return 32 * WT * (dma ? 128 : kLeftPitchPadded) + Tile<T>::BK * 32 * WT * (int)sizeof(T);
}

template <typename T, int WT, bool DMA> struct TileStaging {
    static constexpr int BM = 32 * WT, BN = 32 * WT;
    static constexpr int BK = Tile<T>::BK, VN = Tile<T>::VN;
    static constexpr int APitch = DMA ? 128 : kLeftPitchPadded;
    static constexpr int BPitch = BN * (int)sizeof(T);   // right rows are rotated, not padded
    static constexpr int KQ = BK / 4;                    // k values each 16-lane group owns per k-block
    static constexpr int VPR = BN / VN;                  // 16-byte vectors per right row
    static constexpr int BSTEP = kTileThreads / VPR;     // right rows covered by one pass of the workgroup
    static constexpr int kRot = 16 * (int)sizeof(T);     // rotation of a right row per k-group, in bytes
    static constexpr int kLeftBytes = BM * APitch;       // the right tile starts here
    static_assert(BK / BSTEP == WT && BM / 32 == WT, "WT staged vectors per thread and operand");

    // vector v = tid + 256 i of a tile: left row = tid / 8 + 32 i, right row = tid / VPR + BSTEP i
    int a_row0, a_col;   // left: first row and the element column of this thread's vectors (register staging)
    int b_row0, b_col;   // right: first row and element column
    int a_lds, b_lds;    // byte offsets of the thread's first left / right vector in a stage (register staging)
    int b_vcol;          // byte offset of the thread's vector inside an unrotated right row
    int a_kv;            // direct-to-LDS: element offset of the k-vector that belongs in this thread's left slot
    int slot_base;       // direct-to-LDS: byte offset of this wave's 64 slots inside one pass (wave-uniform)
    int vslot;           // tid % VPR

    __device__ __forceinline__ explicit TileStaging(int tid)
    {
        a_row0 = tid >> 3;
        a_col = (tid & 7) * VN;
        b_row0 = tid / VPR;
        vslot = tid % VPR;
        b_col = vslot * VN;
        a_lds = a_row0 * APitch + (tid & 7) * 16;
        b_lds = kLeftBytes + b_row0 * BPitch;
        b_vcol = vslot * 16;
        a_kv = ((tid & 7) ^ ((tid >> 4) & 7)) * VN;   // ((row / 2) & 7) does not depend on the pass
        slot_base = __builtin_amdgcn_readfirstlane(tid >> 6) * 64 * 16;
    }
    // register staging: byte offset of staged left / right vector i
    __device__ __forceinline__ int left_write(int i) const { return a_lds + 32 * i * APitch; }
    __device__ __forceinline__ int right_write(int i) const
    {
        return b_lds + BSTEP * i * BPitch + ((b_vcol + kRot * ((b_row0 + BSTEP * i) / KQ)) & (BPitch - 1));
    }
    // direct-to-LDS: row of the left / right tile this thread's slot of pass i lies in, the element column of the
    // right vector that belongs there, and the slot's byte offset inside its tile
    __device__ __forceinline__ int left_row(int i) const { return a_row0 + 32 * i; }
    __device__ __forceinline__ int right_row(int i) const { return b_row0 + BSTEP * i; }
    __device__ __forceinline__ int right_col(int i) const
    {
        return ((vslot - (kRot / 16) * (right_row(i) / KQ)) & (VPR - 1)) * VN;
    }
    __device__ __forceinline__ int slot(int i) const { return i * 256 * 16 + slot_base; }
    // Fetch one k-block straight into `stage`: left rows lrow0.. of L (leading dimension ldl) at inner index k0..,
    // right rows k0.. of R (leading dimension ldr) at columns col0.. .  Every access must be in bounds.
    __device__ __forceinline__ void fetch_to_lds(const T *L, size_t ldl, int lrow0, const T *R, size_t ldr, int col0, int k0,
                                                 unsigned char *stage) const
    {
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            const T *ga = L + (size_t)(lrow0 + left_row(i)) * ldl + k0 + a_kv;
            const T *gb = R + (size_t)(k0 + right_row(i)) * ldr + col0 + right_col(i);
            to_lds(ga, stage + slot(i));
            to_lds(gb, stage + kLeftBytes + slot(i));
        }
    }
    // The same for one side only: the left tile to `dst`, or the right tile to `dst`.
    __device__ __forceinline__ void fetch_left_to_lds(const T *L, size_t ldl, int lrow0, int k0, unsigned char *dst) const
    {
#pragma unroll
        for (int i = 0; i < WT; ++i) to_lds(L + (size_t)(lrow0 + left_row(i)) * ldl + k0 + a_kv, dst + slot(i));
    }
    __device__ __forceinline__ void fetch_right_to_lds(const T *R, size_t ldr, int col0, int k0, unsigned char *dst) const
    {
#pragma unroll
        for (int i = 0; i < WT; ++i) to_lds(R + (size_t)(k0 + right_row(i)) * ldr + col0 + right_col(i), dst + slot(i));
    }
    static __device__ __forceinline__ void to_lds(const T *g, unsigned char *lds)
    {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                         (__attribute__((address_space(3))) void *)lds, 16, 0, 0);
    }
    // Fragment reads of wave (wm, wn), lane (lg = lane / 16, lj = lane % 16):
    //   left: row (wm 16 WT + 16 ti + lj), k values lg KQ .. lg KQ + KQ - 1 -> two 16-byte reads (h = 0, 1) at
    //         left_read(wm, lj, lg, h) + ti 16 APitch
    //   right: row (lg KQ + kk) at right_read_base(lg) + kk BPitch, columns rotated by 16 lg elements
    static __device__ __forceinline__ int left_read(int wm, int lj, int lg, int h)
    {
        const int row = (wm * 16 * WT + lj) * APitch;
        return row + (DMA ? ((2 * lg + h) ^ ((lj >> 1) & 7)) * 16 : lg * 32 + 16 * h);
    }
    static __device__ __forceinline__ int right_read_base(int lg) { return kLeftBytes + (lg * KQ) * BPitch; }
    static constexpr int kRightBytes = BK * BPitch;
};

}  // namespace expmk
