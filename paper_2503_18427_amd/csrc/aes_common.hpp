// Shared host-side plumbing of the gfx950 AES-SpMM library: error reporting,
// argument checks, launch helpers.  Device code lives in the .hip files.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "aes_spmm.h"

namespace aes {

constexpr int kWave = 64;          // gfx950 wavefront width
constexpr int kBlock = 256;        // threads per workgroup used by every kernel here
constexpr int kWavesPerBlock = kBlock / kWave;

// 16-byte and 4-byte accesses that assume only the alignment of one element (4 bytes for float32
// rows, 1 byte for rows of 8-bit codes): gfx950 global memory instructions accept them, and the
// compiler still emits one dwordx4 / dword instruction, so leading dimensions and base addresses
// need no padding; an unaligned row merely touches at most one more 128-byte line.
struct __attribute__((packed, aligned(4))) Float4U { float x, y, z, w; };
struct __attribute__((packed, aligned(1))) Word1U { uint32_t v; };

// Thread-local message of the last failing call.
char *error_buffer();
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(AES_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return AES_OK;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// AES_Q_PER_ROW_INLINE: a node's constants live in its own row of codes, the float32 scale at byte
// q_inline_offset(F) (the codes rounded up to a multiple of four), the affine scheme's zero point in
// the four bytes after it.  Checks the layout and returns where node 0's constants are and how many
// floats lie between two nodes' constants.
inline int64_t q_inline_offset(int32_t F) { return (static_cast<int64_t>(F) + 3) & ~static_cast<int64_t>(3); }

inline int q_inline_constants(const char *what, const int8_t *Xq, int64_t ldq, int32_t F, bool affine,
                              const float *&scale, const float *&zero, int64_t &stride)
{
    const int64_t off = q_inline_offset(F), need = off + (affine ? 8 : 4);
    if (ldq < need || ldq % 4 != 0)
        return fail(AES_ERR_INVALID_ARG, "%s: constants inside the rows need ldq >= %lld and a multiple of 4 (ldq=%lld, F=%d)",
                    what, (long long)need, (long long)ldq, (int)F);
    if (!aligned(Xq, 4)) return fail(AES_ERR_INVALID_ARG, "%s: constants inside the rows need Xq 4-byte aligned", what);
    scale = reinterpret_cast<const float *>(Xq + off);
    zero = affine ? scale + 1 : nullptr;
    stride = ldq / 4;
    return AES_OK;
}

// Smallest power of two >= v (v >= 1).
inline int pow2_ceil(int64_t v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace aes
