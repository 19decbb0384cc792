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

// Smallest power of two >= v (v >= 1).
inline int pow2_ceil(int64_t v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace aes
