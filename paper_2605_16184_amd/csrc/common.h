// Host-side helpers shared by the entry points: argument checks, workspace carving and the
// asynchronous host -> device table upload.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#include "../../include/asteria.h"

namespace asteria {

#define ASTERIA_HIP_TRY(expr)                          \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return ASTERIA_HIP_ERROR; \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Sequential carving of a caller-owned workspace into 256-byte aligned pieces.
struct Carver {
    unsigned char *base;
    size_t off;
    explicit Carver(void *p) : base(reinterpret_cast<unsigned char *>(p)), off(0) {}
    template <typename T> T *take(size_t count)
    {
        T *p = reinterpret_cast<T *>(base + off);
        off += align_up(count * sizeof(T), 256);
        return p;
    }
    static size_t need(size_t count, size_t elem) { return align_up(count * elem, 256); }
};

// Host -> device copy that is ordered on the stream, never blocks and never reads host memory
// after it returns: the bytes travel as by-value kernel arguments, one chunk per launch.
constexpr int UPLOAD_WORDS = 896;   // 3584 bytes per launch, below the 4 KiB argument limit
struct UploadChunk { uint32_t w[UPLOAD_WORDS]; };

static __global__ void upload_chunk_kernel(uint32_t *dst, UploadChunk chunk, int nwords)
{
    for (int i = threadIdx.x; i < nwords; i += blockDim.x) dst[i] = chunk.w[i];
}

// dst must be 4-byte aligned; bytes is rounded up to whole words (dst needs that much room).
inline hipError_t upload_async(void *dst, const void *src, size_t bytes, hipStream_t stream)
{
    const size_t nwords = (bytes + 3) / 4;
    const unsigned char *s = reinterpret_cast<const unsigned char *>(src);
    uint32_t *d = reinterpret_cast<uint32_t *>(dst);
    size_t done = 0;
    while (done < nwords) {
        const size_t n = (nwords - done < (size_t)UPLOAD_WORDS) ? (nwords - done) : (size_t)UPLOAD_WORDS;
        UploadChunk c;
        const size_t byte_off = done * 4;
        const size_t nbytes = (bytes - byte_off < n * 4) ? (bytes - byte_off) : n * 4;
        memset(&c, 0, sizeof(uint32_t) * n);
        memcpy(&c, s + byte_off, nbytes);
        hipLaunchKernelGGL(upload_chunk_kernel, dim3(1), dim3(256), 0, stream, d + done, c, (int)n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        done += n;
    }
    return hipSuccess;
}

inline bool valid_dtype(int d) { return d == ASTERIA_F32 || d == ASTERIA_BF16; }

}  // namespace asteria
