// Device-side addressing shared by the kernels of libftp (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ftp {

constexpr int kTabGrid = 16;

// Where the map of one boundary lives and how a stack addresses it.  A whole (group-boundary) map
// has stack stride 0 and origin (0,0); a per-stack slot starts at the stack's own rectangle.
struct View {
    void* p;
    long long ss, ns, cs;         // element strides: stack, image, channel
    int pitch;                    // elements per row
    int x0[kTabGrid], y0[kTabGrid];   // map coordinate of the slot origin, per tile column / row
};

// Rectangle each stack works on: x interval per tile column, y interval per tile row (inclusive).
struct RectTab {
    int x0[kTabGrid], x1[kTabGrid], y0[kTabGrid], y1[kTabGrid];
};

typedef uint16_t bf16_t;          // raw bfloat16 bits

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
// fp32 -> bfloat, nearest with ties to even: the conversion instruction of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t bf16_bits(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)v); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16_t* p, float v) { *p = (bf16_t)bf16_bits(v); }

// Value a map element holds after being stored with element type T (identity for fp32).
__device__ __forceinline__ float stored(float v, const float*) { return v; }
__device__ __forceinline__ float stored(float v, const bf16_t*) { return __uint_as_float(bf16_bits(v) << 16); }

template <typename T>
__device__ __forceinline__ T* at(const View& v, int stack, int ti, int tj, int n, int c, int y, int x)
{
    return (T*)v.p + (long long)stack * v.ss + (long long)n * v.ns + (long long)c * v.cs +
           (long long)(y - v.y0[ti]) * v.pitch + (x - v.x0[tj]);
}

// The dispatcher hands the workgroups of a launch to the 8 XCDs round-robin by linear index, and every XCD has an L2 of
// its own.  Kernels in which a group of `gx` workgroups reads the same maps launch a 1-D grid of
// 8 * gx * ceil(groups / 8) workgroups and number them so that a group's workgroups run on one XCD, one after the
// other, while consecutive groups go to different XCDs (so uneven groups still spread over the chip):
// XCD x = index % 8 works through the groups x, x + 8, x + 16, ...  Returns false for the padding (group >= groups).
__device__ __forceinline__ bool xcd_order(int groups, int gx, int& group, int& block)
{
    const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3;
    const int round = slot / gx;
    block = slot - round * gx;
    group = xcd + 8 * round;
    return group < groups;
}
inline unsigned xcd_grid(int groups, int gx) { return (unsigned)(8 * gx * ((groups + 7) / 8)); }

// Value of lane (lane ^ X) for X = 1, 2, 3: an exchange inside a quad of lanes, done by the vector ALU's data-parallel
// primitives (quad_perm), not by a round trip through the LDS crossbar.
template <int X>
__device__ __forceinline__ float quad_xor(float v)
{
    constexpr int ctrl = X == 1 ? 0xB1 : X == 2 ? 0x4E : 0x1B;          // quad_perm [1,0,3,2] / [2,3,0,1] / [3,2,1,0]
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), ctrl, 0xF, 0xF, true));
}

__device__ __forceinline__ float leaky(float z, float slope) { return z > 0.0f ? z : slope * z; }

// Packed activation signs of a boundary (whole map): bit c % 32 of the 32-bit word [image][c / 32][y][x] is set
// where the activation of channel c is > 0.
__device__ __forceinline__ uint32_t sign_bit(const View& sg, int stack, int ti, int tj, int n, int c, int y, int x)
{
    return (*at<uint32_t>(sg, stack, ti, tj, n, c >> 5, y, x) >> (c & 31)) & 1u;
}

// What a pass writes into the delta map of a boundary that carries an activation: dLoss/dY, rounded as a map of
// type T holds it, times the leaky-ReLU derivative there (1 where the activation is positive, else slope).
template <typename T>
__device__ __forceinline__ float scaled_delta(float v, uint32_t positive, float slope)
{
    const float r = stored(v, (const T*)nullptr);
    return positive ? r : slope * r;
}

}  // namespace ftp
